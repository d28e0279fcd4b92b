// Bandwidth-bound kernels: element-wise maps, row reductions, the generic one-output-per-lane EinSum
// and the aggregation of partial slabs.
//
// Paper passages: the unary / element-wise forms of EinSum and the softmax pieces are Section 3; the
// per-block kernel K (the inner EinSum on one pair of sub-tensors) is Section 4.3; the aggregation
// operator (group by the surviving key, reduce with (+)) is Section 4.2.  One launch covers every
// tuple of the join: the workgroup index selects (tuple, piece of that tuple's block).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "eg_device.h"

namespace eg {

constexpr int kThreads = 256;

__device__ __forceinline__ char *out_base(const OutSpec &o, int64_t agg)
{
    // partial mode: slab aggIdx of the fp32 workspace; otherwise the destination tensor itself
    return (char *)o.ptr + (o.slab_elems ? agg * o.slab_elems * 4 : 0);
}

// ------------------------------------------------------------------------------------------------
// generic EinSum: one output element per lane, sequential fp32 loop over the aggregated labels.
// A sum is accumulated with a compensation term (Kahan): one lane may add up tens of thousands of
// same-signed terms, and plain sequential fp32 addition would then lose more than the 1e-5 the
// fp32 results are held to; the compensated sum's error does not grow with the number of terms.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_generic(const GenericParams p)
{
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= p.n_tuples * p.outs_per_block) return;
    const int64_t t = gid / p.outs_per_block, e = gid - t * p.outs_per_block;
    int64_t ox, oy, oz, agg;
    decode_tuple(p.ts, t, ox, oy, oz, agg);
    decode_dims(p.zdims, e, ox, oy, oz);
    float acc = oplus_identity(p.oplus);
    const int nr = p.rdims.n;
    if (nr == 0) {
        float x = load_elem(p.x, p.dtx, ox);
        float y = p.binary ? load_elem(p.y, p.dty, oy) : 0.f;
        acc = oplus_eval(p.oplus, acc, otimes_eval(p.otimes, x, y, p.alpha));
    } else {
        int32_t idx[kMaxDims];
        for (int i = 0; i < kMaxDims; i++) idx[i] = 0;
        const int last = nr - 1;
        const int64_t lsx = p.rdims.sx[last], lsy = p.rdims.sy[last];
        const int32_t ln = p.rdims.ext[last];
        const int64_t outer = p.red_elems / ln;
        float comp = 0.f;
        for (int64_t it = 0; it < outer; it++) {
            int64_t bx = ox, by = oy;
            for (int i = 0; i < last; i++) {
                bx += (int64_t)idx[i] * p.rdims.sx[i];
                by += (int64_t)idx[i] * p.rdims.sy[i];
            }
            for (int32_t r = 0; r < ln; r++) {
                float x = load_elem(p.x, p.dtx, bx + r * lsx);
                float y = p.binary ? load_elem(p.y, p.dty, by + r * lsy) : 0.f;
                const float v = otimes_eval(p.otimes, x, y, p.alpha);
                if (p.oplus == EG_AGG_SUM) {
                    const float u = v - comp, s = acc + u;
                    comp = (s - acc) - u;
                    acc = s;
                } else {
                    acc = oplus_eval(p.oplus, acc, v);
                }
            }
            for (int i = last - 1; i >= 0; i--) {
                if (++idx[i] < p.rdims.ext[i]) break;
                idx[i] = 0;
            }
        }
    }
    store_elem(out_base(p.out, agg), p.out.dtype, oz, acc);
}

// ------------------------------------------------------------------------------------------------
// element-wise map / binary join without aggregated labels; VEC elements per lane along the last dim.
// grid.x covers one tuple's block (one vector per lane: many small workgroups stream best from HBM),
// grid.y/z select the tuple, so everything about the tuple is scalar work.
// ------------------------------------------------------------------------------------------------
// grid.x is the tuple and grid.y/z the position inside the tuple's block, so workgroups that start together work at
// the same position of neighbouring blocks: where the blocks cut the innermost label, that is one contiguous stretch
// of every operand instead of short row pieces a whole row apart (+34 % on a map over rows cut eight ways).
__device__ __forceinline__ int64_t tuple_of_block() { return (int64_t)blockIdx.x; }
__device__ __forceinline__ uint32_t pos_of_block() { return blockIdx.z * gridDim.y + blockIdx.y; }

// Every lane decodes its own flat index in the block and handles one vector.  (A variant that kept a workgroup inside
// one long row, four vectors per lane and the row's offsets as scalar work, was 8 % slower once the workgroups ran
// tuple-interleaved: 5.2 against 5.6-5.7 TB/s on 180 MB operands.)
template <int VEC, int OP, bool FAST>
__global__ __launch_bounds__(kThreads) void k_map(const MapParams p)
{
    const int64_t t = tuple_of_block();
    const uint32_t pos = pos_of_block();
    int64_t ox, oy, oz, agg;
    decode_tuple(p.ts, t, ox, oy, oz, agg);
    const int vd = p.dims.n - 1;
    const uint32_t nv = ((uint32_t)p.dims.ext[vd] + VEC - 1) / VEC;
    const uint32_t e0 = pos * kThreads + threadIdx.x;
    if (pos >= ((uint32_t)p.vecs_per_block + kThreads - 1) / kThreads || e0 >= (uint32_t)p.vecs_per_block) return;
    uint32_t e = e0 / nv;
    const uint32_t col = e0 - e * nv;
    for (int i = vd - 1; i >= 0; i--) {
        const uint32_t ext = (uint32_t)p.dims.ext[i], q = e / ext;
        const int64_t k2 = e - q * ext;
        e = q;
        ox += k2 * p.dims.sx[i]; oy += k2 * p.dims.sy[i]; oz += k2 * p.dims.sz[i];
    }
    char *zb = out_base(p.out, agg);
    if (VEC == 8 && (int64_t)col * VEC + VEC > p.dims.ext[vd]) {
        // the last, partial vector of a dense one-dimensional index space (any other space has whole vectors only)
        for (int64_t k = (int64_t)col * VEC; k < p.dims.ext[vd]; k++) {
            const float x = load_elem(p.x, p.dtx, ox + k * p.dims.sx[vd]);
            const float y = p.binary ? load_elem(p.y, p.dty, oy + k * p.dims.sy[vd]) : 0.f;
            store_elem(zb, p.out.dtype, oz + k * p.dims.sz[vd], otimes_t<OP, FAST>(p.otimes, x, y, p.alpha));
        }
    } else if (VEC == 8) {
        float x[8], y[8], z[8];
        const int64_t k = (int64_t)col * VEC;
        if (p.dims.sx[vd] == 1) load8(p.x, p.dtx, ox + k, x);
        else { float s = load_elem(p.x, p.dtx, ox + k * p.dims.sx[vd]);
#pragma unroll
            for (int i = 0; i < 8; i++) x[i] = s; }
        if (p.binary) {
            if (p.dims.sy[vd] == 1) load8(p.y, p.dty, oy + k, y);
            else { float s = load_elem(p.y, p.dty, oy + k * p.dims.sy[vd]);
#pragma unroll
                for (int i = 0; i < 8; i++) y[i] = s; }
        } else {
#pragma unroll
            for (int i = 0; i < 8; i++) y[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; i++) z[i] = otimes_t<OP, FAST>(p.otimes, x[i], y[i], p.alpha);
        store8(zb, p.out.dtype, oz + k * p.dims.sz[vd], z);
    } else {
        const int64_t k = col;
        float x = load_elem(p.x, p.dtx, ox + k * p.dims.sx[vd]);
        float y = p.binary ? load_elem(p.y, p.dty, oy + k * p.dims.sy[vd]) : 0.f;
        store_elem(zb, p.out.dtype, oz + k * p.dims.sz[vd], otimes_t<OP, FAST>(p.otimes, x, y, p.alpha));
    }
}

// Element-wise vertex with one transposed operand (`ij->ji`, `bhst->bhts`, `ij,ji->ij`): Z is contiguous along its
// last dimension a = dims[n-1], the transposed operand T along another one, b = dims[td].  A workgroup moves a tile of
// 64 (a) x 64 (b): T is read in 16-byte vectors along b into LDS (as fp32, rows padded to 65 words), then every
// lane gathers 8 consecutive a for one b from LDS, reads the other operand (if any) along Z, and writes a 16-byte
// vector of Z.  Element by element these vertices ran at 1.0-1.6 TB/s.
constexpr int kTrTile = 64;

template <int OP, bool FAST>
__global__ __launch_bounds__(kThreads) void k_map_tr(const MapParams p)
{
    __shared__ float tile[kTrTile][kTrTile + 1];
    const int64_t t = tuple_of_block();
    uint32_t pos = pos_of_block();
    const int vd = p.dims.n - 1, td = p.td;
    const uint32_t ea = (uint32_t)p.dims.ext[vd], eb = (uint32_t)p.dims.ext[td];
    const uint32_t ta = (ea + kTrTile - 1) / kTrTile, tb = (eb + kTrTile - 1) / kTrTile;
    const bool xt = p.tr == 1;                                      // which operand is the transposed one
    const int64_t *st = xt ? p.dims.sx : p.dims.sy, *so = xt ? p.dims.sy : p.dims.sx;
    int64_t ox, oy, oz, agg;
    decode_tuple(p.ts, t, ox, oy, oz, agg);
    int64_t ot = xt ? ox : oy, oo = xt ? oy : ox;
    const uint32_t b0 = (pos % tb) * kTrTile;
    pos /= tb;
    const uint32_t a0 = (pos % ta) * kTrTile;
    pos /= ta;
    for (int i = vd - 1; i >= 0; i--) {
        if (i == td) continue;
        const uint32_t ext = (uint32_t)p.dims.ext[i], q = pos / ext;
        const int64_t k = pos - q * ext;
        pos = q;
        ot += k * st[i]; oo += k * so[i]; oz += k * p.dims.sz[i];
    }
    if (pos != 0) return;                                           // beyond the block (whole workgroups leave)
    const void *tp = xt ? p.x : p.y, *op = xt ? p.y : p.x;
    const int dtt = xt ? p.dtx : p.dty, dto = xt ? p.dty : p.dtx;
#pragma unroll
    for (int h = 0; h < kTrTile * kTrTile / 8 / kThreads; h++) {    // T: rows along a, vectors along b
        const int v = h * kThreads + threadIdx.x, ra = v / (kTrTile / 8), vb = v % (kTrTile / 8);
        if (a0 + ra < ea && b0 + vb * 8 < eb) {
            float x[8];
            load8(tp, dtt, ot + (int64_t)(a0 + ra) * st[vd] + (b0 + vb * 8), x);
#pragma unroll
            for (int i = 0; i < 8; i++) tile[ra][vb * 8 + i] = x[i];
        }
    }
    __syncthreads();
    char *zb = out_base(p.out, agg);
#pragma unroll
    for (int h = 0; h < kTrTile * kTrTile / 8 / kThreads; h++) {    // Z: rows along b, vectors along a
        const int v = h * kThreads + threadIdx.x, rb = v / (kTrTile / 8), va = v % (kTrTile / 8);
        if (b0 + rb < eb && a0 + va * 8 < ea) {
            float tv[8], ov[8], z[8];
#pragma unroll
            for (int i = 0; i < 8; i++) tv[i] = tile[va * 8 + i][rb];
            if (p.binary) {
                const int64_t o = oo + (int64_t)(b0 + rb) * so[td] + (int64_t)(a0 + va * 8) * so[vd];
                if (so[vd] == 1) load8(op, dto, o, ov);
                else { const float sv = load_elem(op, dto, o);
#pragma unroll
                    for (int i = 0; i < 8; i++) ov[i] = sv; }
            } else {
#pragma unroll
                for (int i = 0; i < 8; i++) ov[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < 8; i++) z[i] = otimes_t<OP, FAST>(p.otimes, xt ? tv[i] : ov[i], xt ? ov[i] : tv[i], p.alpha);
            store8(zb, p.out.dtype, oz + (int64_t)(b0 + rb) * p.dims.sz[td] + (a0 + va * 8), z);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// row reduction: LANES lanes cooperate on one output element; the reduced labels are X's trailing dims.
// With split > 1 (few outputs, long reductions) each output's reduction range is cut into `split` pieces
// that land in consecutive partial slabs (slab = aggIdx * split + piece) for the aggregation kernel.
// ------------------------------------------------------------------------------------------------
template <int OPLUS, int GROUP = 64>                     // over aligned groups of GROUP lanes (a power of two)
__device__ __forceinline__ float wave_reduce(int oplus, float v)
{
#pragma unroll
    for (int off = GROUP / 2; off >= 1; off >>= 1) v = oplus_t<OPLUS>(oplus, v, __shfl_xor(v, off, 64));
    return v;
}

// LANES lanes share one output (8 .. 64: several outputs per wave, short rows; 256: one per workgroup); U vectors
// per lane are loaded before any is used (1 where a lane has a single vector anyway).
template <int LANES, int VEC, int OP, int OPLUS, int U>
__global__ __launch_bounds__(kThreads) void k_reduce_row(const ReduceParams p)
{
    constexpr int PER_WG = kThreads / LANES;
    __shared__ float red[kThreads / 64];
    const int sub = threadIdx.x / LANES, lane = threadIdx.x % LANES;
    const int64_t t = tuple_of_block();
    const uint32_t slot = pos_of_block() * PER_WG + sub;              // (output, piece) within the tuple's block
    const uint32_t split = (uint32_t)p.split;
    const uint32_t o = slot / split, piece = slot - o * split;
    const bool active = t < p.n_tuples && o < (uint32_t)p.outs_per_block;   // whole lane groups are active or not
    float acc = oplus_identity(OPLUS >= 0 ? OPLUS : p.oplus);
    int64_t oz = 0, agg = 0;
    if (active) {
        int64_t ox, oy;
        decode_tuple(p.ts, t, ox, oy, oz, agg);
        {
            uint32_t e = o;
            for (int i = p.zdims.n - 1; i >= 0; i--) {
                const uint32_t ext = (uint32_t)p.zdims.ext[i], q = e / ext;
                const int64_t k = e - q * ext;
                e = q;
                ox += k * p.zdims.sx[i]; oy += k * p.zdims.sy[i]; oz += k * p.zdims.sz[i];
            }
        }
        const int vd = p.rdims.n - 1;
        const uint32_t nv = ((uint32_t)p.rdims.ext[vd] + VEC - 1) / VEC;
        const uint32_t total = (uint32_t)(p.red_elems / p.rdims.ext[vd]) * nv;
        const uint32_t chunk = (total + split - 1) / split;
        const uint32_t lo = piece * chunk, hi = (lo + chunk < total) ? lo + chunk : total;
        const bool flat = p.rdims.n == 1;
        for (uint32_t j0 = lo + lane; j0 < hi; j0 += U * LANES) {
            float x[U][VEC], y[U][VEC];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; u++) {                          // issue the loads of U vectors before using any
                const uint32_t j = j0 + u * LANES;
                ok[u] = j < hi;
                const uint32_t jj = ok[u] ? j : lo;
                int64_t bx, by;
                if (flat) {
                    bx = ox + (int64_t)jj * VEC * p.rdims.sx[vd];
                    by = oy + (int64_t)jj * VEC * p.rdims.sy[vd];
                } else {
                    uint32_t q = jj / nv;
                    const int64_t k = (int64_t)(jj - q * nv) * VEC;
                    bx = ox + k * p.rdims.sx[vd];
                    by = oy + k * p.rdims.sy[vd];
                    for (int i = vd - 1; i >= 0; i--) {
                        const uint32_t ext = (uint32_t)p.rdims.ext[i], q2 = q / ext;
                        const int64_t k2 = q - q2 * ext;
                        q = q2;
                        bx += k2 * p.rdims.sx[i]; by += k2 * p.rdims.sy[i];
                    }
                }
                if (VEC == 8) {
                    load8(p.x, p.dtx, bx, (float (&)[8])x[u]);
                    if (p.binary) {
                        if (p.rdims.sy[vd] == 1) load8(p.y, p.dty, by, (float (&)[8])y[u]);
                        else { float s = load_elem(p.y, p.dty, by);
#pragma unroll
                            for (int i = 0; i < VEC; i++) y[u][i] = s; }
                    }
                } else {
                    x[u][0] = load_elem(p.x, p.dtx, bx);
                    if (p.binary) y[u][0] = load_elem(p.y, p.dty, by);
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                if (!ok[u]) continue;
#pragma unroll
                for (int i = 0; i < VEC; i++)
                    acc = oplus_t<OPLUS>(p.oplus, acc, otimes_t<OP, false>(p.otimes, x[u][i], p.binary ? y[u][i] : 0.f, p.alpha));
            }
        }
    }
    acc = wave_reduce<OPLUS, (LANES < 64 ? LANES : 64)>(p.oplus, acc);
    // partial mode: slab (aggIdx * split + piece) of the fp32 workspace; otherwise the destination tensor
    char *zb = (char *)p.out.ptr + (p.out.slab_elems ? (agg * split + piece) * p.out.slab_elems * 4 : 0);
    if (LANES > 64) {                       // one output per workgroup: combine the four waves through LDS
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            float v = red[0];
            for (int w = 1; w < kThreads / 64; w++) v = oplus_t<OPLUS>(p.oplus, v, red[w]);
            if (active) store_elem(zb, p.out.dtype, oz, v);
        }
    } else if (lane == 0 && active) {
        store_elem(zb, p.out.dtype, oz, acc);
    }
}

// Short rows: an (output, piece) has at most LANES vectors, one per lane, and a group of LANES lanes takes R
// consecutive ones, loading all R vectors before it reduces any.  A wave that held a single kilobyte in flight and
// then walked through its cross-lane reduction left the memory system idle most of the time (0.6 TB/s on rows of 128
// elements, 2.4 on rows of 512; with this 4-5 TB/s).
template <int LANES, int OP, int OPLUS, int R>
__global__ __launch_bounds__(kThreads) void k_reduce_short(const ReduceParams p)
{
    constexpr int PER_WG = kThreads / LANES, VEC = 8;
    const int sub = threadIdx.x / LANES, lane = threadIdx.x % LANES;
    const int64_t t = tuple_of_block();
    const uint32_t slot0 = (pos_of_block() * PER_WG + sub) * R;
    const uint32_t split = (uint32_t)p.split;
    int64_t tx, ty, tz, agg;
    decode_tuple(p.ts, t, tx, ty, tz, agg);
    const int vd = p.rdims.n - 1;
    const uint32_t nv = ((uint32_t)p.rdims.ext[vd] + VEC - 1) / VEC;
    const uint32_t total = (uint32_t)(p.red_elems / p.rdims.ext[vd]) * nv;
    const uint32_t chunk = (total + split - 1) / split;
    float x[R][VEC], y[R][VEC];
    bool act[R], ok[R];
    int64_t oz[R];
    uint32_t piece[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        const uint32_t slot = slot0 + r;
        uint32_t o = slot / split;
        piece[r] = slot - o * split;
        act[r] = o < (uint32_t)p.outs_per_block;
        int64_t ox = tx, oy = ty;
        oz[r] = tz;
        uint32_t e = act[r] ? o : 0;
        for (int i = p.zdims.n - 1; i >= 0; i--) {
            const uint32_t ext = (uint32_t)p.zdims.ext[i], q = e / ext;
            const int64_t k = e - q * ext;
            e = q;
            ox += k * p.zdims.sx[i]; oy += k * p.zdims.sy[i]; oz[r] += k * p.zdims.sz[i];
        }
        const uint32_t lo = piece[r] * chunk, hi = (lo + chunk < total) ? lo + chunk : total;
        const uint32_t j = lo + lane;
        ok[r] = act[r] && j < hi;
        if (ok[r]) {
            uint32_t q = j / nv;
            const int64_t k = (int64_t)(j - q * nv) * VEC;
            int64_t bx = ox + k * p.rdims.sx[vd], by = oy + k * p.rdims.sy[vd];
            for (int i = vd - 1; i >= 0; i--) {
                const uint32_t ext = (uint32_t)p.rdims.ext[i], q2 = q / ext;
                const int64_t k2 = q - q2 * ext;
                q = q2;
                bx += k2 * p.rdims.sx[i]; by += k2 * p.rdims.sy[i];
            }
            load8(p.x, p.dtx, bx, x[r]);
            if (p.binary) {
                if (p.rdims.sy[vd] == 1) load8(p.y, p.dty, by, y[r]);
                else { const float sv = load_elem(p.y, p.dty, by);
#pragma unroll
                    for (int i = 0; i < VEC; i++) y[r][i] = sv; }
            }
        }
    }
    float acc[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        acc[r] = oplus_identity(OPLUS >= 0 ? OPLUS : p.oplus);
        if (ok[r]) {
#pragma unroll
            for (int i = 0; i < VEC; i++)
                acc[r] = oplus_t<OPLUS>(p.oplus, acc[r], otimes_t<OP, false>(p.otimes, x[r][i], p.binary ? y[r][i] : 0.f, p.alpha));
        }
    }
#pragma unroll
    for (int off = LANES / 2; off >= 1; off >>= 1) {
#pragma unroll
        for (int r = 0; r < R; r++) acc[r] = oplus_t<OPLUS>(p.oplus, acc[r], __shfl_xor(acc[r], off, 64));
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < R; r++) {
            if (!act[r]) continue;
            char *zb = (char *)p.out.ptr + (p.out.slab_elems ? (agg * split + piece[r]) * p.out.slab_elems * 4 : 0);
            store_elem(zb, p.out.dtype, oz[r], acc[r]);
        }
    }
}

// Reduction over labels that lie outside the outputs' innermost dimension (column sums, `ij->j`, `bij->bj`,
// `ij,ij->j`): that dimension has stride 1 in X and Z, so a lane owns 8 consecutive outputs and walks a part of the
// reduced index space, four 16-byte loads in flight.  A workgroup covers a strip of 32 output vectors (512 contiguous
// bytes of bf16 per step) with 8 lane groups that split the piece's range [lo, hi) into 8 consecutive parts and are
// combined through LDS in ascending order; the pieces (one per workgroup and strip) become partial slabs like those
// of a split row reduction.  Sums carry a compensation term, as in the one-output-per-lane kernel: a lane may add
// tens of thousands of same-signed terms.
constexpr int kColStrip = 32, kColGroups = kThreads / kColStrip;

template <int OP, int OPLUS>
__global__ __launch_bounds__(kThreads) void k_reduce_col(const ReduceParams p)
{
    constexpr int VEC = 8, U = 4;
    __shared__ float part[kColGroups][kColStrip][VEC + 1];
    const int64_t t = tuple_of_block();
    const int zd = p.zdims.n - 1;
    const uint32_t nvz = (uint32_t)p.zdims.ext[zd] / VEC;
    const uint32_t vecs = (uint32_t)(p.outs_per_block / VEC), split = (uint32_t)p.split;
    const uint32_t strips = (vecs + kColStrip - 1) / kColStrip;
    const uint32_t wg = pos_of_block();
    if (wg >= strips * split) return;                               // whole workgroups leave
    const uint32_t piece = wg / strips, strip = wg - piece * strips;
    const int lv = threadIdx.x % kColStrip, grp = threadIdx.x / kColStrip;
    const uint32_t ov = strip * kColStrip + lv;
    const bool active = ov < vecs;
    int64_t ox, oy, oz, agg;
    decode_tuple(p.ts, t, ox, oy, oz, agg);
    {
        uint32_t e = (active ? ov : 0) / nvz;
        const int64_t c = (int64_t)((active ? ov : 0) - e * nvz) * VEC;
        ox += c * p.zdims.sx[zd]; oz += c; oy += c * p.zdims.sy[zd];
        for (int i = zd - 1; i >= 0; i--) {
            const uint32_t ext = (uint32_t)p.zdims.ext[i], q = e / ext;
            const int64_t k = e - q * ext;
            e = q;
            ox += k * p.zdims.sx[i]; oy += k * p.zdims.sy[i]; oz += k * p.zdims.sz[i];
        }
    }
    const uint32_t total = (uint32_t)p.red_elems, chunk = (total + split - 1) / split;
    const uint32_t plo = piece * chunk, phi = (plo + chunk < total) ? plo + chunk : total;
    const uint32_t sub = (phi - plo + kColGroups - 1) / kColGroups;
    const uint32_t lo = plo + grp * sub < phi ? plo + grp * sub : phi, hi = (lo + sub < phi) ? lo + sub : phi;
    const bool sum = (OPLUS >= 0 ? OPLUS : p.oplus) == EG_AGG_SUM;
    const bool xvec = p.zdims.sx[zd] == 1, yvec = p.binary && p.zdims.sy[zd] == 1;   // else one value for the 8 outputs
    const int rl = p.rdims.n - 1;
    float acc[VEC], comp[VEC];
#pragma unroll
    for (int i = 0; i < VEC; i++) { acc[i] = oplus_identity(OPLUS >= 0 ? OPLUS : p.oplus); comp[i] = 0.f; }
    for (uint32_t j0 = lo; active && j0 < hi; j0 += U) {
        float x[U][VEC], y[U][VEC];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const uint32_t j = j0 + u < hi ? j0 + u : lo;           // a valid position; its values are not used
            uint32_t q = j / (uint32_t)p.rdims.ext[rl];
            const int64_t k = j - q * (uint32_t)p.rdims.ext[rl];
            int64_t bx = ox + k * p.rdims.sx[rl], by = oy + k * p.rdims.sy[rl];
            for (int i = rl - 1; i >= 0; i--) {
                const uint32_t ext = (uint32_t)p.rdims.ext[i], q2 = q / ext;
                const int64_t k2 = q - q2 * ext;
                q = q2;
                bx += k2 * p.rdims.sx[i]; by += k2 * p.rdims.sy[i];
            }
            if (xvec) load8(p.x, p.dtx, bx, x[u]);
            else { const float sv = load_elem(p.x, p.dtx, bx);
#pragma unroll
                for (int i = 0; i < VEC; i++) x[u][i] = sv; }
            if (yvec) load8(p.y, p.dty, by, y[u]);
            else if (p.binary) { const float sv = load_elem(p.y, p.dty, by);
#pragma unroll
                for (int i = 0; i < VEC; i++) y[u][i] = sv; }
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (j0 + u >= hi) continue;
#pragma unroll
            for (int i = 0; i < VEC; i++) {
                const float v = otimes_t<OP, false>(p.otimes, x[u][i], p.binary ? y[u][i] : 0.f, p.alpha);
                if (sum) {
                    const float d = v - comp[i], s2 = acc[i] + d;
                    comp[i] = (s2 - acc[i]) - d;
                    acc[i] = s2;
                } else {
                    acc[i] = oplus_t<OPLUS>(p.oplus, acc[i], v);
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < VEC; i++) part[grp][lv][i] = acc[i];
    __syncthreads();
    if (grp != 0 || !active) return;
#pragma unroll
    for (int g = 1; g < kColGroups; g++) {                         // ascending parts; an empty part holds the identity
#pragma unroll
        for (int i = 0; i < VEC; i++) acc[i] = oplus_t<OPLUS>(p.oplus, acc[i], part[g][lv][i]);
    }
    char *zb = (char *)p.out.ptr + (p.out.slab_elems ? (agg * split + piece) * p.out.slab_elems * 4 : 0);
    store8(zb, p.out.dtype, oz, acc);
}

// ------------------------------------------------------------------------------------------------
// aggregation of partial slabs: out[e] = (+)_{a ascending} partials[a][e], fp32, one final cast
// ------------------------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));

// N > 0: the slab count is known at compile time, so all N loads are in flight before the first add.
// The adds themselves stay in ascending slab order.  Partial slabs are read once: streaming loads.
template <int N>
__global__ __launch_bounds__(kThreads) void k_aggregate_vec4(const AggregateParams p)
{
    const int64_t i4 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t e = i4 * 4;
    if (e >= p.slab_elems) return;
    const f32x4 *src = (const f32x4 *)(p.partials + e);
    const int64_t slab4 = p.slab_stride / 4;
    f32x4 acc;
    if (N > 0) {
        f32x4 v[N > 0 ? N : 1];
#pragma unroll
        for (int a = 0; a < N; a++) v[a] = __builtin_nontemporal_load(src + a * slab4);
        acc = v[0];
#pragma unroll
        for (int a = 1; a < N; a++) {
            if (p.oplus == EG_AGG_MAX) { acc.x = fmaxf(acc.x, v[a].x); acc.y = fmaxf(acc.y, v[a].y); acc.z = fmaxf(acc.z, v[a].z); acc.w = fmaxf(acc.w, v[a].w); }
            else acc += v[a];
        }
    } else {
        acc = __builtin_nontemporal_load(src);
        if (p.oplus == EG_AGG_MAX) {
#pragma unroll 4
            for (int64_t a = 1; a < p.n_agg; a++) {
                f32x4 v = __builtin_nontemporal_load(src + a * slab4);
                acc.x = fmaxf(acc.x, v.x); acc.y = fmaxf(acc.y, v.y); acc.z = fmaxf(acc.z, v.z); acc.w = fmaxf(acc.w, v.w);
            }
        } else {
#pragma unroll 4
            for (int64_t a = 1; a < p.n_agg; a++) acc += __builtin_nontemporal_load(src + a * slab4);
        }
    }
    if (p.out_dtype == EG_BF16) {
        uint2 r;
        r.x = pack_bf16x2(acc.x, acc.y);
        r.y = pack_bf16x2(acc.z, acc.w);
        *(uint2 *)((uint16_t *)p.out + e) = r;
    } else {
        *(f32x4 *)((float *)p.out + e) = acc;
    }
}

__global__ __launch_bounds__(kThreads) void k_aggregate_scalar(const AggregateParams p)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= p.slab_elems) return;
    // ascending slab order, eight loads in flight at a time (a loss cut into hundreds of pieces is one such chain)
    float acc = p.partials[e];
    for (int64_t a = 1; a < p.n_agg; a += 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) v[j] = p.partials[(a + j < p.n_agg ? a + j : a) * p.slab_stride + e];
#pragma unroll
        for (int j = 0; j < 8; j++)
            if (a + j < p.n_agg) acc = oplus_eval(p.oplus, acc, v[j]);
    }
    int64_t off = e;
    if (!p.contiguous) {
        int64_t ox = 0, oy = 0;
        off = 0;
        decode_dims(p.dims, e, ox, oy, off);
    }
    store_elem(p.out, p.out_dtype, off, acc);
}

// Few outputs, many slabs (a loss whose reduction was cut into hundreds of pieces): one wave per output element.
// The lanes fetch 512 slabs' values at once into LDS; one lane then adds them one after the other in ascending slab
// order, so the result is that of the plain loop (reading a value from another lane's register for every addition
// instead cost 35 ns per slab).
__global__ __launch_bounds__(64) void k_aggregate_wave(const AggregateParams p)
{
    constexpr int B = 8;
    __shared__ float4 sh[64 * B / 4];
    const int64_t e = blockIdx.x;
    const int lane = threadIdx.x;
    const float ident = oplus_identity(p.oplus);           // x (+) identity = x exactly, so the chain may start from it
    float acc = ident;
    for (int64_t a0 = 0; a0 < p.n_agg; a0 += 64 * B) {
        float v[B];
#pragma unroll
        for (int b = 0; b < B; b++) {
            const int64_t a = a0 + b * 64 + lane;
            v[b] = a < p.n_agg ? p.partials[a * p.slab_stride + e] : ident;
        }
        __syncthreads();                                   // the previous round's values have been read
#pragma unroll
        for (int b = 0; b < B; b++) ((float *)sh)[b * 64 + lane] = v[b];
        __syncthreads();
        if (lane == 0) {
            const int64_t left = p.n_agg - a0;
            const int cnt = (int)(left < 64 * B ? left : 64 * B);
            // slots past cnt hold the identity (see the fill above), so whole vectors are added
            if (p.oplus == EG_AGG_MAX) {
                for (int j = 0; j < cnt; j += 4) { const float4 q = sh[j / 4]; acc = fmaxf(fmaxf(fmaxf(fmaxf(acc, q.x), q.y), q.z), q.w); }
            } else {
                for (int j = 0; j < cnt; j += 4) { const float4 q = sh[j / 4]; acc = (((acc + q.x) + q.y) + q.z) + q.w; }
            }
        }
    }
    if (lane != 0) return;
    int64_t off = e;
    if (!p.contiguous) {
        int64_t ox = 0, oy = 0;
        off = 0;
        decode_dims(p.dims, e, ox, oy, off);
    }
    store_elem(p.out, p.out_dtype, off, acc);
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
static int grid_for(int64_t items, int64_t per_wg, unsigned &grid)
{
    int64_t g = (items + per_wg - 1) / per_wg;
    if (g < 1) g = 1;
    if (g >= (1ll << 31)) return fail(EG_ERR_LIMIT, "launch needs %lld workgroups", (long long)g);
    grid = (unsigned)g;
    return EG_OK;
}

static int check_launch(const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "%s launch failed: %s", what, hipGetErrorString(e));
    return EG_OK;
}

int launch_generic(const GenericParams &p, void *stream)
{
    if (!p.x || (p.binary && !p.y) || !p.out.ptr) return fail(EG_ERR_NULL, "generic kernel: NULL operand");
    if (p.n_tuples >= (1ll << 31)) return fail(EG_ERR_LIMIT, "too many tuples");
    unsigned grid;
    int rc = grid_for(p.n_tuples * p.outs_per_block, kThreads, grid);
    if (rc) return rc;
    EG_LAUNCH(k_generic, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return check_launch("k_generic");
}

// grid.x = tuples, grid.y * grid.z >= workgroups per tuple (y at most 65535, z as small as that allows)
static int tuple_grid(int64_t per_tuple_items, int64_t per_wg, int64_t n_tuples, dim3 &grid)
{
    int64_t g = (per_tuple_items + per_wg - 1) / per_wg;
    if (g < 1) g = 1;
    if (g >= (1ll << 31) || per_tuple_items >= (1ll << 32)) return fail(EG_ERR_LIMIT, "block too large for one launch");
    if (n_tuples >= (1ll << 31)) return fail(EG_ERR_LIMIT, "too many tuples");
    const int64_t gz = (g + 65534) / 65535;
    const int64_t gy = (g + gz - 1) / gz;              // at most gz - 1 workgroups beyond g
    grid = dim3((unsigned)n_tuples, (unsigned)gy, (unsigned)gz);
    return EG_OK;
}

template <int OP>
static void launch_map_vec(const MapParams &p, dim3 grid, hipStream_t st)
{
    const bool fast = p.out.dtype == EG_BF16;     // hardware exponential only where the result is rounded to bf16
    if (fast) EG_LAUNCH((k_map<8, OP, true>), grid, dim3(kThreads), 0, st, p);
    else EG_LAUNCH((k_map<8, OP, false>), grid, dim3(kThreads), 0, st, p);
}

template <int OP>
static void launch_map_tr(const MapParams &p, dim3 grid, hipStream_t st)
{
    if (p.out.dtype == EG_BF16) EG_LAUNCH((k_map_tr<OP, true>), grid, dim3(kThreads), 0, st, p);
    else EG_LAUNCH((k_map_tr<OP, false>), grid, dim3(kThreads), 0, st, p);
}

int launch_map(const MapParams &p, void *stream)
{
    if (!p.x || (p.binary && !p.y) || !p.out.ptr) return fail(EG_ERR_NULL, "map kernel: NULL operand");
    if (p.dims.n < 1) return fail(EG_ERR_LIMIT, "map kernel: empty index space");
    if (p.vec != 1 && p.vec != 8) return fail(EG_ERR_LIMIT, "map kernel: vector width %d", p.vec);
    hipStream_t st = (hipStream_t)stream;
    dim3 grid;
    if (p.tr) {
        const int vd = p.dims.n - 1;
        const int64_t *s = p.tr == 1 ? p.dims.sx : p.dims.sy;
        if ((p.tr != 1 && !(p.tr == 2 && p.binary)) || p.dims.n < 2 || p.td < 0 || p.td >= vd || s[p.td] != 1 || p.dims.sz[vd] != 1 ||
            p.dims.ext[vd] % 8 || p.dims.ext[p.td] % 8)
            return fail(EG_ERR_LIMIT, "map kernel: not a transposed operand");
        int64_t tiles = ((p.dims.ext[vd] + kTrTile - 1) / kTrTile) * ((p.dims.ext[p.td] + kTrTile - 1) / kTrTile);
        for (int i = 0; i < vd; i++)
            if (i != p.td) tiles *= p.dims.ext[i];
        int rc = tuple_grid(tiles, 1, p.n_tuples, grid);
        if (rc) return rc;
        switch (p.otimes) {
#define EG_CASE(OP) case OP: launch_map_tr<OP>(p, grid, st); break;
        EG_CASE(EG_MUL) EG_CASE(EG_ADD) EG_CASE(EG_SUB) EG_CASE(EG_IDENT) EG_CASE(EG_SCALE)
#undef EG_CASE
        default: launch_map_tr<-1>(p, grid, st); break;
        }
        return check_launch("k_map_tr");
    }
    int rc = tuple_grid(p.vecs_per_block, kThreads, p.n_tuples, grid);
    if (rc) return rc;
    if (p.vec == 1) {
        EG_LAUNCH((k_map<1, -1, false>), grid, dim3(kThreads), 0, st, p);
        return check_launch("k_map");
    }
    switch (p.otimes) {
#define EG_CASE(OP) case OP: launch_map_vec<OP>(p, grid, st); break;
    EG_CASE(EG_MUL) EG_CASE(EG_ADD) EG_CASE(EG_SUB) EG_CASE(EG_DIV) EG_CASE(EG_SQDIFF) EG_CASE(EG_ABSDIFF)
    EG_CASE(EG_EXP_SUB) EG_CASE(EG_RELU_GRAD) EG_CASE(EG_SILU_MUL) EG_CASE(EG_IDENT) EG_CASE(EG_SCALE)
    EG_CASE(EG_RELU) EG_CASE(EG_EXP) EG_CASE(EG_LOG)
#undef EG_CASE
    default: return fail(EG_ERR_BAD_OP, "map kernel: unknown scalar function %d", p.otimes);
    }
    return check_launch("k_map");
}

template <int LANES, int R>
static void launch_reduce_short(const ReduceParams &p, dim3 grid, hipStream_t st)
{
    if (p.otimes == EG_IDENT && p.oplus == EG_AGG_MAX) EG_LAUNCH((k_reduce_short<LANES, EG_IDENT, EG_AGG_MAX, R>), grid, dim3(kThreads), 0, st, p);
    else if (p.otimes == EG_IDENT && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_short<LANES, EG_IDENT, EG_AGG_SUM, R>), grid, dim3(kThreads), 0, st, p);
    else if (p.otimes == EG_MUL && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_short<LANES, EG_MUL, EG_AGG_SUM, R>), grid, dim3(kThreads), 0, st, p);
    else EG_LAUNCH((k_reduce_short<LANES, -1, -1, R>), grid, dim3(kThreads), 0, st, p);
}

template <int LANES, int VEC, int U>
static void launch_reduce_ops(const ReduceParams &p, dim3 grid, hipStream_t st)
{
    // the common (x)/(+) pairs are compiled in; anything else reads them at run time
    if (p.otimes == EG_IDENT && p.oplus == EG_AGG_MAX) EG_LAUNCH((k_reduce_row<LANES, VEC, EG_IDENT, EG_AGG_MAX, U>), grid, dim3(kThreads), 0, st, p);
    else if (p.otimes == EG_IDENT && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_row<LANES, VEC, EG_IDENT, EG_AGG_SUM, U>), grid, dim3(kThreads), 0, st, p);
    else if (p.otimes == EG_MUL && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_row<LANES, VEC, EG_MUL, EG_AGG_SUM, U>), grid, dim3(kThreads), 0, st, p);
    else EG_LAUNCH((k_reduce_row<LANES, VEC, -1, -1, U>), grid, dim3(kThreads), 0, st, p);
}

int launch_reduce_row(const ReduceParams &p, void *stream)
{
    if (!p.x || (p.binary && !p.y) || !p.out.ptr) return fail(EG_ERR_NULL, "reduce kernel: NULL operand");
    if (p.rdims.n < 1) return fail(EG_ERR_LIMIT, "reduce kernel: empty reduction space");
    if (p.split < 1 || (p.split > 1 && !p.out.slab_elems)) return fail(EG_ERR_LIMIT, "reduce kernel: split needs partial slabs");
    if (p.red_elems >= (1ll << 32)) return fail(EG_ERR_LIMIT, "reduce kernel: reduction space above 2^32");
    hipStream_t st = (hipStream_t)stream;
    if (p.col) {
        const int zd = p.zdims.n - 1;
        if (p.zdims.n < 1 || p.zdims.ext[zd] % 8 || (p.zdims.sx[zd] != 1 && p.zdims.sx[zd] != 0) || p.zdims.sz[zd] != 1 || p.outs_per_block % 8)
            return fail(EG_ERR_LIMIT, "reduce kernel: outputs are not whole 16-byte vectors");
        dim3 grid;
        int rc = tuple_grid((p.outs_per_block / 8 + kColStrip - 1) / kColStrip * p.split, 1, p.n_tuples, grid);
        if (rc) return rc;
        if (p.otimes == EG_IDENT && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_col<EG_IDENT, EG_AGG_SUM>), grid, dim3(kThreads), 0, st, p);
        else if (p.otimes == EG_IDENT && p.oplus == EG_AGG_MAX) EG_LAUNCH((k_reduce_col<EG_IDENT, EG_AGG_MAX>), grid, dim3(kThreads), 0, st, p);
        else if (p.otimes == EG_MUL && p.oplus == EG_AGG_SUM) EG_LAUNCH((k_reduce_col<EG_MUL, EG_AGG_SUM>), grid, dim3(kThreads), 0, st, p);
        else EG_LAUNCH((k_reduce_col<-1, -1>), grid, dim3(kThreads), 0, st, p);
        return check_launch("k_reduce_col");
    }
    const int64_t slots = p.outs_per_block * p.split;
    // vectors one (output, piece) reduces over, as the kernel counts them
    const int vd = p.rdims.n - 1;
    const int64_t total = (p.red_elems / p.rdims.ext[vd]) * ((p.rdims.ext[vd] + p.vec - 1) / p.vec);
    const int64_t chunk = (total + p.split - 1) / p.split;
    const bool wide = chunk * p.vec >= 16384 || slots * p.n_tuples < 1024;   // long or few rows: a workgroup each
    int lanes = 256;
    if (!wide) {
        lanes = 64;
        if (p.vec == 8) while (lanes > 8 && lanes / 2 >= chunk) lanes /= 2;   // short rows: several outputs per wave
    }
    dim3 grid;
    if (p.vec == 8 && lanes <= 64 && chunk <= lanes) {        // one vector per lane: four (output, piece) per lane group
        constexpr int R = 4;
        int rc = tuple_grid(slots, kThreads / lanes * R, p.n_tuples, grid);
        if (rc) return rc;
        if (lanes == 64) launch_reduce_short<64, R>(p, grid, st);
        else if (lanes == 32) launch_reduce_short<32, R>(p, grid, st);
        else if (lanes == 16) launch_reduce_short<16, R>(p, grid, st);
        else launch_reduce_short<8, R>(p, grid, st);
        return check_launch("k_reduce_short");
    }
    int rc = tuple_grid(slots, kThreads / lanes, p.n_tuples, grid);
    if (rc) return rc;
    if (p.vec == 8) {
        if (lanes == 256) launch_reduce_ops<256, 8, 4>(p, grid, st);
        else launch_reduce_ops<64, 8, 4>(p, grid, st);
    } else {
        if (lanes == 256) launch_reduce_ops<256, 1, 4>(p, grid, st);
        else launch_reduce_ops<64, 1, 4>(p, grid, st);
    }
    return check_launch("k_reduce_row");
}

int launch_aggregate(const AggregateParams &p, void *stream)
{
    if (!p.partials || !p.out) return fail(EG_ERR_NULL, "aggregate kernel: NULL operand");
    if (p.n_agg < 1 || p.slab_elems < 1) return fail(EG_ERR_LIMIT, "aggregate kernel: empty input");
    if (p.slab_stride < p.slab_elems) return fail(EG_ERR_LIMIT, "aggregate kernel: slabs overlap");
    const bool vec = p.contiguous && p.slab_elems % 4 == 0 && p.slab_stride % 4 == 0 && ((uintptr_t)p.partials & 15) == 0 &&
                     ((uintptr_t)p.out & 15) == 0;
    unsigned grid;
    if (p.n_agg >= 32 && p.slab_elems <= 4096) {                    // too few outputs for one lane per output to hide the loads
        EG_LAUNCH(k_aggregate_wave, dim3((unsigned)p.slab_elems), dim3(64), 0, (hipStream_t)stream, p);
        return check_launch("k_aggregate");
    }
    int rc = grid_for(vec ? p.slab_elems / 4 : p.slab_elems, kThreads, grid);
    if (rc) return rc;
    if (vec) {
        hipStream_t st = (hipStream_t)stream;
        switch (p.n_agg) {
        case 2: EG_LAUNCH(k_aggregate_vec4<2>, dim3(grid), dim3(kThreads), 0, st, p); break;
        case 4: EG_LAUNCH(k_aggregate_vec4<4>, dim3(grid), dim3(kThreads), 0, st, p); break;
        case 8: EG_LAUNCH(k_aggregate_vec4<8>, dim3(grid), dim3(kThreads), 0, st, p); break;
        case 16: EG_LAUNCH(k_aggregate_vec4<16>, dim3(grid), dim3(kThreads), 0, st, p); break;
        default: EG_LAUNCH(k_aggregate_vec4<0>, dim3(grid), dim3(kThreads), 0, st, p); break;
        }
    } else EG_LAUNCH(k_aggregate_scalar, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return check_launch("k_aggregate");
}

}  // namespace eg

// ------------------------------------------------------------------------------------------------
// Fused softmax over the last label (Section 3 of the paper gives softmax as row maximum, exp(x - maximum),
// row sum and division; here the four run as one pass per row, with the preceding alpha * x + y when there is
// one).  Values are rounded where the separate vertices would have rounded (dt_t after the addition, dt_e
// after the exponential), so the result matches the unfused path up to the order of the row sum.
// ------------------------------------------------------------------------------------------------
namespace eg {

__device__ __forceinline__ float round_as(float v, int dt) { return dt == EG_BF16 ? bf16_to_f32(f32_to_bf16(v)) : v; }

__device__ __forceinline__ void softmax_row_offsets(const SoftmaxParams &p, int64_t t, uint32_t row, int64_t &ox, int64_t &oy, int64_t &oz, int64_t &oc, int64_t &os)
{
    int64_t unused0, unused1;
    decode_tuple(p.ts, t, ox, oy, oz, unused0);
    decode_tuple(p.ts2, t, oc, os, unused0, unused1);
    uint32_t e = row;
    for (int i = p.rows.n - 1; i >= 0; i--) {
        const uint32_t ext = (uint32_t)p.rows.ext[i], q = e / ext;
        const int64_t k = e - q * ext;
        e = q;
        ox += k * p.rows.sx[i]; oy += k * p.rows.sy[i]; oz += k * p.rows.sz[i];
        oc += k * p.stats.sx[i]; os += k * p.stats.sy[i];
    }
}

// Element offsets of the row in the tensors that tails bring (read: entries 0, 1; written by tail k: 2 + k).  One walk over the
// tuple's and the row's keys for all entries, so that an iteration's stride loads go out together.
__device__ __forceinline__ void softmax_more_offsets(const SoftmaxParams &p, int64_t t, uint32_t row, int64_t (&o)[kSoftmaxMore])
{
#pragma unroll
    for (int e = 0; e < kSoftmaxMore; e++) o[e] = 0;
    uint32_t rem = (uint32_t)t;
    for (int l = p.ts.n - 1; l >= 0; l--) {
        const uint32_t dd = (uint32_t)p.ts.d[l], q = rem / dd;
        const int64_t k = rem - q * dd;
        rem = q;
#pragma unroll
        for (int e = 0; e < kSoftmaxMore; e++) o[e] += k * p.more_step[e][l];
    }
    uint32_t r = row;
    for (int i = p.rows.n - 1; i >= 0; i--) {
        const uint32_t ext = (uint32_t)p.rows.ext[i], q = r / ext;
        const int64_t k = r - q * ext;
        r = q;
#pragma unroll
        for (int e = 0; e < kSoftmaxMore; e++) o[e] += k * p.more_rows[e][i];
    }
}

// A tail's scalar function as its own vertex would evaluate it (hardware exponential and reciprocal where the result is
// stored as bf16), rounded to the vertex's dtype.
__device__ __noinline__ float softmax_tail_eval(int op, float alpha, int dt, float a, float b)
{
    const float v = dt == EG_BF16 ? otimes_t<-1, true>(op, a, b, alpha) : otimes_t<-1, false>(op, a, b, alpha);
    return round_as(v, dt);
}

// The same for the 8 elements of a lane's vector.  One copy of the code for all tails and vectors (a call, not inlined: inlined
// into every tail of every vector the scalar functions' switch made a kernel of 45 000 instructions that ran four times as long).
typedef float f32x8 __attribute__((ext_vector_type(8)));
__device__ __noinline__ f32x8 softmax_tail_eval8(int op, float alpha, int dt, f32x8 a, f32x8 b)
{
    f32x8 r;
    if (dt == EG_BF16) {
#pragma unroll
        for (int i = 0; i < 8; i++) r[i] = otimes_t<-1, true>(op, a[i], b[i], alpha);
#pragma unroll
        for (int i = 0; i < 8; i += 2) { float x = r[i], y = r[i + 1]; round_pair_bf16(x, y); r[i] = x; r[i + 1] = y; }
    } else {
#pragma unroll
        for (int i = 0; i < 8; i++) r[i] = otimes_t<-1, false>(op, a[i], b[i], alpha);
    }
    return r;
}

// A pass's tail descriptors in registers: read from the kernel arguments once, all loads issued together (read where they
// are used, every access was a scalar load of its own with its own wait, some hundred per wave, and the pass took 60 us
// on rows that the chain alone covers in 15).
struct SoftmaxTailRegs {
    int op[kSoftmaxTails], a[kSoftmaxTails], b[kSoftmaxTails], row[kSoftmaxTails], dt[kSoftmaxTails], emit[kSoftmaxTails];
    float alpha[kSoftmaxTails];
    void *out[kSoftmaxTails];
    const void *ext[kSoftmaxExt];
    int dt_ext[kSoftmaxExt];
    int n_tail, n_ext;
};
__device__ __forceinline__ void softmax_tail_regs(const SoftmaxParams &p, SoftmaxTailRegs &r)
{
    r.n_tail = p.n_tail; r.n_ext = p.n_ext;
#pragma unroll
    for (int k = 0; k < kSoftmaxTails; k++) {
        r.op[k] = p.tail[k].op; r.a[k] = p.tail[k].a; r.b[k] = p.tail[k].b; r.row[k] = p.tail[k].row;
        r.dt[k] = p.tail[k].dt; r.emit[k] = p.tail[k].emit; r.alpha[k] = p.tail[k].alpha; r.out[k] = p.tail[k].out;
    }
    // the values are wanted here, in scalar registers: keeps the compiler from moving each load to its first use
#pragma unroll
    for (int k = 0; k < kSoftmaxTails; k++) {
        asm volatile("" : "+s"(r.op[k]), "+s"(r.a[k]), "+s"(r.b[k]), "+s"(r.row[k]), "+s"(r.dt[k]), "+s"(r.emit[k]), "+s"(r.alpha[k]), "+s"(r.out[k]));
    }
#pragma unroll
    for (int e = 0; e < kSoftmaxExt; e++) {
        r.ext[e] = p.ext[e]; r.dt_ext[e] = p.dt_ext[e];
        asm volatile("" : "+s"(r.ext[e]), "+s"(r.dt_ext[e]));
    }
    asm volatile("" : "+s"(r.n_tail), "+s"(r.n_ext));
}

// The per-row tails (operands: the row maximum, the row sum, earlier per-row tails), evaluated by every lane alike.
__device__ __forceinline__ void softmax_row_tails(const SoftmaxTailRegs &td, float m, float sum, float (&rowv)[kSoftmaxTails])
{
#pragma unroll
    for (int k = 0; k < kSoftmaxTails; k++) {
        rowv[k] = 0.f;
        if (k < td.n_tail && td.row[k]) {
            auto slot = [&](int s) {
                switch (s) {
                case 1: return m;
                case 3: return sum;
                case 8: return rowv[0];
                case 9: return rowv[1];
                case 10: return rowv[2];
                default: return 0.f;
                }
            };
            rowv[k] = softmax_tail_eval(td.op[k], td.alpha[k], td.dt[k], slot(td.a[k]), td.b[k] >= 0 ? slot(td.b[k]) : 0.f);
        }
    }
}

template <int U, int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (U < N) {
        f(std::integral_constant<int, U>{});
        static_for<U + 1, N>(f);
    }
}

// One wave per row, VPL vectors of 8 elements per lane held in registers (rows of up to 512 * VPL elements).
// MODE fixes the storage dtypes of the chain at compile time (0: sum, exponentials and result all bf16; 1: all
// fp32; 2: read from the parameters): with run-time dtypes every element pays for both variants of each step.
template <int VPL, int MODE, bool TAIL>
__global__ __launch_bounds__(kThreads) void k_softmax_rows(const SoftmaxParams p)
{
    static_assert(!TAIL || MODE == 2, "tails come with run-time dtypes");
    const int dt_t = MODE == 0 ? EG_BF16 : MODE == 1 ? EG_F32 : p.dt_t;
    const int dt_e = MODE == 0 ? EG_BF16 : MODE == 1 ? EG_F32 : p.dt_e;
    const int dt_p = MODE == 0 ? EG_BF16 : MODE == 1 ? EG_F32 : p.dt_p;
    const int dt_src = MODE == 0 ? EG_BF16 : MODE == 1 ? EG_F32 : p.dt_src;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t t = tuple_of_block();
    const uint32_t row = pos_of_block() * (kThreads / 64) + wave;
    if (t >= p.n_tuples || row >= (uint32_t)p.rows_per_block) return;          // whole waves leave
    int64_t ox, oy, oz, oc, os;
    softmax_row_offsets(p, t, row, ox, oy, oz, oc, os);
    // When the workgroup's rows all take the same row of the added operand (a mask shared by batch entries and
    // heads), the workgroup fetches it once into LDS instead of once per wave.
    __shared__ uint4 addrow[VPL * 128];                 // 512 * VPL elements of up to 4 bytes
    if (p.share_add) {
        const int es = p.dt_add == EG_BF16 ? 2 : 4, chunks = p.n * es / 16;
        const uint4 *g = (const uint4 *)((const char *)p.add + oy * es);
#pragma unroll
        for (int j = 0; j < (VPL + 1) / 2; j++) { const int c = j * kThreads + threadIdx.x; if (c < chunks) addrow[c] = g[c]; }
        __syncthreads();
    }
    float v[VPL][8];
    float tsrc[TAIL ? VPL : 1][8];                      // the chain's source values, for tails that read them
    float m = -INFINITY;
#pragma unroll
    for (int u = 0; u < VPL; u++) {
        const int c = (u * 64 + lane) * 8;
        if (c < p.n) {
            load8(p.src, dt_src, ox + c, v[u]);
            if (p.has_add) {
                float y[8];
                if (p.share_add) load8(addrow, p.dt_add, c, y);
                else if (p.sy_last == 1) load8(p.add, p.dt_add, oy + c, y);
                else { const float s = load_elem(p.add, p.dt_add, oy);
#pragma unroll
                    for (int i = 0; i < 8; i++) y[i] = s; }
#pragma unroll
                for (int i = 0; i < 8; i++) v[u][i] = p.alpha * v[u][i] + y[i];
                if (dt_t == EG_BF16) {
#pragma unroll
                    for (int i = 0; i < 8; i += 2) round_pair_bf16(v[u][i], v[u][i + 1]);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; i++) m = fmaxf(m, v[u][i]);
            if (TAIL) {
#pragma unroll
                for (int i = 0; i < 8; i++) tsrc[u][i] = v[u][i];
            }
        }
    }
    m = round_as(wave_reduce<EG_AGG_MAX>(EG_AGG_MAX, m), p.dt_max);       // the exponentials see the maximum as its vertex stores it
    const bool fast_e = dt_e == EG_BF16, fast_p = dt_p == EG_BF16;         // as the separate vertices choose
    const float neg_m_log2e = -(m * kLog2e);
    float sum = 0.f;
#pragma unroll
    for (int u = 0; u < VPL; u++) {
        if ((u * 64 + lane) * 8 < p.n) {
#pragma unroll
            for (int i = 0; i < 8; i++) v[u][i] = fast_e ? exp_sub_scaled(v[u][i], neg_m_log2e) : expf(v[u][i] - m);
            if (dt_e == EG_BF16) {
#pragma unroll
                for (int i = 0; i < 8; i += 2) round_pair_bf16(v[u][i], v[u][i + 1]);
            }
#pragma unroll
            for (int i = 0; i < 8; i++) sum += v[u][i];
        }
    }
    sum = round_as(wave_reduce<EG_AGG_SUM>(EG_AGG_SUM, sum), p.dt_sum);   // ... and the division the sum as its vertex stores it
    const float inv = __frcp_rn(sum);
    float rowv[kSoftmaxTails];
    int64_t omore[kSoftmaxMore];
    SoftmaxTailRegs td;
    if (TAIL) {
        static_assert(kSoftmaxMore == 6 && kSoftmaxExt == 2, "one statement per entry: the array must stay in registers");
        softmax_tail_regs(p, td);
        softmax_row_tails(td, m, sum, rowv);
        softmax_more_offsets(p, t, row, omore);
    }
    // (unrolled by recursion over the vector's index: with the tails inside, the loop form was left rolled, and its arrays went to scratch memory)
    static_for<0, VPL>([&](auto U) {
        constexpr int u = decltype(U)::value;
        const int c = (u * 64 + lane) * 8;
        if (c < p.n) {
            float z[8];
#pragma unroll
            for (int i = 0; i < 8; i++) z[i] = fast_p ? v[u][i] * inv : v[u][i] / sum;
            if (!TAIL || p.emit_p) store8(p.p, dt_p, oz + c, z);
            if (TAIL) {
                float e0[8], e1[8], tv[kSoftmaxTails][8];
#pragma unroll
                for (int i = 0; i < 8; i++) { e0[i] = e1[i] = 0.f; z[i] = round_as(z[i], dt_p); }      // tails see the quotient as its vertex stores it
                if (td.n_ext > 0) load8(td.ext[0], td.dt_ext[0], omore[0] + c, e0);
                if (td.n_ext > 1) load8(td.ext[1], td.dt_ext[1], omore[1] + c, e1);
                // the 8 values of an operand slot
                auto fetch = [&](int sl, float (&dst)[8]) {
#define EG_SLOT(EXPR) { _Pragma("unroll") for (int i = 0; i < 8; i++) dst[i] = (EXPR); } break
                    switch (sl) {
                    case 0: EG_SLOT(tsrc[TAIL ? u : 0][i]);
                    case 1: EG_SLOT(m);
                    case 2: EG_SLOT(v[u][i]);
                    case 3: EG_SLOT(sum);
                    case 4: EG_SLOT(z[i]);
                    case 5: EG_SLOT(e0[i]);
                    case 6: EG_SLOT(e1[i]);
                    case 8: EG_SLOT(td.row[0] ? rowv[0] : tv[0][i]);
                    case 9: EG_SLOT(td.row[1] ? rowv[1] : tv[1][i]);
                    case 10: EG_SLOT(td.row[2] ? rowv[2] : tv[2][i]);
                    default: EG_SLOT(0.f);
                    }
#undef EG_SLOT
                };
#pragma unroll
                for (int k = 0; k < kSoftmaxTails; k++) {
#pragma unroll
                    for (int i = 0; i < 8; i++) tv[k][i] = 0.f;
                    if (k < td.n_tail && !td.row[k]) {
                        float a[8], b[8];
                        fetch(td.a[k], a);
                        fetch(td.b[k], b);                 // (slot -1: zeros)
                        f32x8 av, bv;
#pragma unroll
                        for (int i = 0; i < 8; i++) { av[i] = a[i]; bv[i] = b[i]; }
                        const f32x8 rv = softmax_tail_eval8(td.op[k], td.alpha[k], td.dt[k], av, bv);
#pragma unroll
                        for (int i = 0; i < 8; i++) tv[k][i] = rv[i];
                        if (td.emit[k]) store8(td.out[k], td.dt[k], omore[2 + k] + c, tv[k]);
                    }
                }
            }
        }
    });
    if (lane == 0) {
        if (p.emit_max) store_elem(p.row_max, p.dt_max, oc, m);
        if (p.emit_sum) store_elem(p.row_sum, p.dt_sum, os, sum);
        if (TAIL) {
#pragma unroll
            for (int k = 0; k < kSoftmaxTails; k++)
                if (k < td.n_tail && td.row[k] && td.emit[k]) store_elem(td.out[k], td.dt[k], omore[2 + k], rowv[k]);
        }
    }
}

// The all-bf16 chain (source, sum in front, exponentials and result stored as bf16) with R consecutive rows per wave: the
// row's offsets are decoded once and advanced by the innermost row label's strides, and the next row's 16-byte loads are
// issued before the current row is worked on, so a wave always has loads in flight (with one row per wave a wave spent
// three quarters of its life waiting: for its scalar loads, then for its row, then for its stores).  Same arithmetic, in the
// same order, as k_softmax_rows<VPL, 0, false>.  The launcher takes it when R divides the innermost row label's extent.
// ADD: 0 no added operand; 1 its row is shared by the workgroup's rows and staged in LDS; 2 read from memory row by row.
// (A template parameter: with the choice made at run time the compiler waited, where the paths meet again, for every load
// in flight, the next row's included.)
template <int VPL, int R, int ADD>
__global__ __launch_bounds__(kThreads) void k_softmax_rows_bf16(const SoftmaxParams p)
{
    typedef uint32_t raw4 __attribute__((ext_vector_type(4)));
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t t = tuple_of_block();
    const uint32_t row0 = (pos_of_block() * (kThreads / 64) + wave) * R;
    if (t >= p.n_tuples || row0 >= (uint32_t)p.rows_per_block) return;         // whole waves leave
    int64_t ox, oy, oz, oc, os;
    softmax_row_offsets(p, t, row0, ox, oy, oz, oc, os);
    const int last = p.rows.n - 1;
    const int64_t dx = p.rows.sx[last], dy = p.rows.sy[last], dz = p.rows.sz[last], dc = p.stats.sx[last], dsum = p.stats.sy[last];
    __shared__ uint4 addrow[ADD == 1 ? VPL * 128 : 1];
    if (ADD == 1) {                                     // one row of the added operand for all rows of the workgroup
        const int es = p.dt_add == EG_BF16 ? 2 : 4, chunks = p.n * es / 16;
        const uint4 *g = (const uint4 *)((const char *)p.add + oy * es);
#pragma unroll
        for (int j = 0; j < (VPL + 1) / 2; j++) { const int c = j * kThreads + threadIdx.x; if (c < chunks) addrow[c] = g[c]; }
    }
    raw4 nxt[VPL];
#pragma unroll
    for (int u = 0; u < VPL; u++) {
        const int c = (u * 64 + lane) * 8;
        if (c < p.n) nxt[u] = *(const raw4 *)((const uint16_t *)p.src + ox + c);
    }
    if (ADD == 1) __syncthreads();
    // A row's results stay in registers until the next row's data has arrived and go out then, in front of the loads of the
    // row after: loads and stores share one in-order counter, and stores issued right before the wait for the next row's
    // data would have to be waited for as well.
    raw4 held[VPL];
    float held_m = 0.f, held_sum = 0.f;
    auto store_row = [&](int j) {
#pragma unroll
        for (int u = 0; u < VPL; u++) {
            const int c = (u * 64 + lane) * 8;
            if (c < p.n) *(raw4 *)((uint16_t *)p.p + oz + j * dz + c) = held[u];
        }
        if (lane == 0) {
            if (p.emit_max) store_elem(p.row_max, p.dt_max, oc + j * dc, held_m);
            if (p.emit_sum) store_elem(p.row_sum, p.dt_sum, os + j * dsum, held_sum);
        }
    };
#pragma unroll
    for (int j = 0; j < R; j++) {
        // this row's data has arrived (and with it everything older); only then the previous row's stores and the next row's loads
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __builtin_amdgcn_sched_barrier(0);
        raw4 cur[VPL];
#pragma unroll
        for (int u = 0; u < VPL; u++) cur[u] = nxt[u];
        if (j > 0) store_row(j - 1);
        __builtin_amdgcn_sched_barrier(0);
        if (j + 1 < R) {
#pragma unroll
            for (int u = 0; u < VPL; u++) {
                const int c = (u * 64 + lane) * 8;
                if (c < p.n) nxt[u] = *(const raw4 *)((const uint16_t *)p.src + ox + (j + 1) * dx + c);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        float v[VPL][8];
        float m = -INFINITY;
#pragma unroll
        for (int u = 0; u < VPL; u++) {
            const int c = (u * 64 + lane) * 8;
            if (c < p.n) {
                const raw4 r = cur[u];
                v[u][0] = __uint_as_float(r.x << 16); v[u][1] = __uint_as_float(r.x & 0xffff0000u);
                v[u][2] = __uint_as_float(r.y << 16); v[u][3] = __uint_as_float(r.y & 0xffff0000u);
                v[u][4] = __uint_as_float(r.z << 16); v[u][5] = __uint_as_float(r.z & 0xffff0000u);
                v[u][6] = __uint_as_float(r.w << 16); v[u][7] = __uint_as_float(r.w & 0xffff0000u);
                if (ADD != 0) {
                    float y[8];
                    if (ADD == 1) load8(addrow, p.dt_add, c, y);
                    else if (p.sy_last == 1) load8(p.add, p.dt_add, oy + j * dy + c, y);
                    else { const float s = load_elem(p.add, p.dt_add, oy + j * dy);
#pragma unroll
                        for (int i = 0; i < 8; i++) y[i] = s; }
#pragma unroll
                    for (int i = 0; i < 8; i++) v[u][i] = p.alpha * v[u][i] + y[i];
#pragma unroll
                    for (int i = 0; i < 8; i += 2) round_pair_bf16(v[u][i], v[u][i + 1]);
                }
#pragma unroll
                for (int i = 0; i < 8; i++) m = fmaxf(m, v[u][i]);
            }
        }
        m = round_as(wave_reduce<EG_AGG_MAX>(EG_AGG_MAX, m), p.dt_max);
        const float neg_m_log2e = -(m * kLog2e);
        float sum = 0.f;
#pragma unroll
        for (int u = 0; u < VPL; u++) {
            if ((u * 64 + lane) * 8 < p.n) {
#pragma unroll
                for (int i = 0; i < 8; i++) v[u][i] = exp_sub_scaled(v[u][i], neg_m_log2e);
#pragma unroll
                for (int i = 0; i < 8; i += 2) round_pair_bf16(v[u][i], v[u][i + 1]);
#pragma unroll
                for (int i = 0; i < 8; i++) sum += v[u][i];
            }
        }
        sum = round_as(wave_reduce<EG_AGG_SUM>(EG_AGG_SUM, sum), p.dt_sum);
        const float inv = __frcp_rn(sum);
#pragma unroll
        for (int u = 0; u < VPL; u++) {
            raw4 o;
            o.x = pack_bf16x2(v[u][0] * inv, v[u][1] * inv); o.y = pack_bf16x2(v[u][2] * inv, v[u][3] * inv);
            o.z = pack_bf16x2(v[u][4] * inv, v[u][5] * inv); o.w = pack_bf16x2(v[u][6] * inv, v[u][7] * inv);
            held[u] = o;
        }
        held_m = m;
        held_sum = sum;
    }
    store_row(R - 1);
}

// Any strides and alignments: one workgroup per row, the row staged in LDS between the three sweeps.
constexpr int kSoftmaxMaxRow = 8192;

__device__ __forceinline__ float block_reduce(float v, int oplus, float *red)
{
    v = oplus == EG_AGG_MAX ? wave_reduce<EG_AGG_MAX>(oplus, v) : wave_reduce<EG_AGG_SUM>(oplus, v);
    __syncthreads();                                   // red[] may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = red[0];
    for (int w = 1; w < kThreads / 64; w++) r = oplus == EG_AGG_MAX ? fmaxf(r, red[w]) : r + red[w];
    return r;
}

__global__ __launch_bounds__(kThreads) void k_softmax_rows_scalar(const SoftmaxParams p)
{
    __shared__ float buf[kSoftmaxMaxRow];
    __shared__ float red[kThreads / 64];
    const int64_t t = tuple_of_block();
    const uint32_t row = pos_of_block();
    if (t >= p.n_tuples || row >= (uint32_t)p.rows_per_block) return;          // whole workgroups leave
    int64_t ox, oy, oz, oc, os;
    softmax_row_offsets(p, t, row, ox, oy, oz, oc, os);
    float m = -INFINITY;
    for (int c = threadIdx.x; c < p.n; c += kThreads) {
        float x = load_elem(p.src, p.dt_src, ox + c * p.sx_last);
        if (p.has_add) x = round_as(p.alpha * x + load_elem(p.add, p.dt_add, oy + c * p.sy_last), p.dt_t);
        buf[c] = x;
        m = fmaxf(m, x);
    }
    m = round_as(block_reduce(m, EG_AGG_MAX, red), p.dt_max);
    const bool fast_e = p.dt_e == EG_BF16, fast_p = p.dt_p == EG_BF16;
    float sum = 0.f;
    for (int c = threadIdx.x; c < p.n; c += kThreads) {
        const float e = round_as(fast_e ? exp_sub_fast(buf[c], m) : expf(buf[c] - m), p.dt_e);
        buf[c] = e;
        sum += e;
    }
    sum = round_as(block_reduce(sum, EG_AGG_SUM, red), p.dt_sum);
    const float inv = __frcp_rn(sum);
    const bool tails = p.n_tail > 0;
    float rowv[kSoftmaxTails];
    int64_t omore[kSoftmaxMore];
    SoftmaxTailRegs td;
    if (tails) {
        softmax_tail_regs(p, td);
        softmax_row_tails(td, m, sum, rowv);
        softmax_more_offsets(p, t, row, omore);
    }
    for (int c = threadIdx.x; c < p.n; c += kThreads) {
        const float q = fast_p ? buf[c] * inv : buf[c] / sum;
        if (p.emit_p) store_elem(p.p, p.dt_p, oz + c * p.sz_last, q);
        if (tails) {
            float x = load_elem(p.src, p.dt_src, ox + c * p.sx_last);                 // the chain's source value, as in the first sweep
            if (p.has_add) x = round_as(p.alpha * x + load_elem(p.add, p.dt_add, oy + c * p.sy_last), p.dt_t);
            const float e0 = td.n_ext > 0 ? load_elem(p.ext[0], p.dt_ext[0], omore[0] + c * p.more_last[0]) : 0.f;
            const float e1 = td.n_ext > 1 ? load_elem(p.ext[1], p.dt_ext[1], omore[1] + c * p.more_last[1]) : 0.f;
            const float qz = round_as(q, p.dt_p);
            float tv[kSoftmaxTails] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < kSoftmaxTails; k++) {
                if (k < td.n_tail && !td.row[k]) {
                    auto slot = [&](int sl) {
                        switch (sl) {
                        case 0: return x;
                        case 1: return m;
                        case 2: return buf[c];
                        case 3: return sum;
                        case 4: return qz;
                        case 5: return e0;
                        case 6: return e1;
                        case 8: return td.row[0] ? rowv[0] : tv[0];
                        case 9: return td.row[1] ? rowv[1] : tv[1];
                        case 10: return td.row[2] ? rowv[2] : tv[2];
                        default: return 0.f;
                        }
                    };
                    tv[k] = softmax_tail_eval(td.op[k], td.alpha[k], td.dt[k], slot(td.a[k]), td.b[k] >= 0 ? slot(td.b[k]) : 0.f);
                    if (td.emit[k]) store_elem(td.out[k], td.dt[k], omore[2 + k] + c * p.more_last[2 + k], tv[k]);
                }
            }
        }
    }
    if (threadIdx.x == 0) {
        if (p.emit_max) store_elem(p.row_max, p.dt_max, oc, m);
        if (p.emit_sum) store_elem(p.row_sum, p.dt_sum, os, sum);
        if (tails) {
#pragma unroll
            for (int k = 0; k < kSoftmaxTails; k++)
                if (k < td.n_tail && td.row[k] && td.emit[k]) store_elem(td.out[k], td.dt[k], omore[2 + k], rowv[k]);
        }
    }
}

int launch_softmax_rows(SoftmaxParams &p, void *stream)
{
    if (!p.src || (p.emit_p && !p.p) || (p.has_add && !p.add) || (p.emit_max && !p.row_max) || (p.emit_sum && !p.row_sum))
        return fail(EG_ERR_NULL, "softmax kernel: NULL operand");
    if (p.n_tail < 0 || p.n_tail > kSoftmaxTails || p.n_ext < 0 || p.n_ext > kSoftmaxExt) return fail(EG_ERR_LIMIT, "softmax kernel: %d tails, %d tensors read by them", p.n_tail, p.n_ext);
    for (int e = 0; e < p.n_ext; e++)
        if (!p.ext[e]) return fail(EG_ERR_NULL, "softmax kernel: NULL operand of a tail");
    for (int k = 0; k < p.n_tail; k++)
        if (p.tail[k].emit && !p.tail[k].out) return fail(EG_ERR_NULL, "softmax kernel: NULL result of a tail");
    if (p.n < 1 || p.n > kSoftmaxMaxRow) return fail(EG_ERR_LIMIT, "softmax kernel: row length %d", p.n);
    if (p.rows_per_block < 1 || p.n_tuples < 1) return fail(EG_ERR_LIMIT, "softmax kernel: empty index space");
    // 16-byte accesses along the rows need unit stride, whole vectors, and every other offset a multiple of 8 elements
    bool vec = p.n % 8 == 0 && p.sx_last == 1 && (!p.emit_p || p.sz_last == 1) && (!p.has_add || p.sy_last == 1 || p.sy_last == 0) &&
               ((uintptr_t)p.src & 15) == 0 && (!p.emit_p || ((uintptr_t)p.p & 15) == 0) && (!p.has_add || ((uintptr_t)p.add & 15) == 0);
    for (int i = 0; i < p.rows.n && vec; i++)
        if (p.rows.sx[i] % 8 || (p.emit_p && p.rows.sz[i] % 8) || (p.has_add && p.sy_last == 1 && p.rows.sy[i] % 8)) vec = false;
    for (int l = 0; l < p.ts.n && vec; l++)
        if (p.ts.step_x[l] % 8 || (p.emit_p && p.ts.step_z[l] % 8) || (p.has_add && p.sy_last == 1 && p.ts.step_y[l] % 8)) vec = false;
    // the tensors of full rank that tails read or write take 16-byte accesses too, or the whole pass goes element by element
    for (int e = 0; e < kSoftmaxMore && vec; e++) {
        const bool used = e < kSoftmaxExt ? e < p.n_ext : (e - kSoftmaxExt < p.n_tail && p.tail[e - kSoftmaxExt].emit && !p.tail[e - kSoftmaxExt].row);
        if (!used) continue;
        const void *q = e < kSoftmaxExt ? p.ext[e] : p.tail[e - kSoftmaxExt].out;
        if (p.more_last[e] != 1 || ((uintptr_t)q & 15)) vec = false;
        for (int i = 0; i < p.rows.n && vec; i++)
            if (p.more_rows[e][i] % 8) vec = false;
        for (int l = 0; l < p.ts.n && vec; l++)
            if (p.more_step[e][l] % 8) vec = false;
    }
    if (p.n_tail > 0 && p.n > 2048) vec = false;      // the register-resident pass carries tails for rows of up to 2048 elements
    p.vec = vec ? 8 : 1;
    // rows of a workgroup are kThreads / 64 consecutive ones; if the innermost row labels that the added operand
    // lacks span a multiple of that many rows, the workgroup's rows share one row of the added operand
    constexpr int rpw = kThreads / 64;
    int64_t lacking = 1;
    for (int i = p.rows.n - 1; i >= 0 && p.rows.sy[i] == 0; i--) lacking *= p.rows.ext[i];
    // the all-bf16 chain on rows of up to 2048 elements, four rows per wave: when the innermost row label holds whole
    // groups of four and every workgroup is full
    constexpr int kRowsPerWave = 4;
    const bool bf16_chain = p.dt_src == EG_BF16 && p.dt_t == EG_BF16 && p.dt_e == EG_BF16 && p.dt_p == EG_BF16;
    const bool multi = vec && bf16_chain && p.n_tail == 0 && p.emit_p && p.n <= 2048 && p.rows.n >= 1 &&
                       p.rows.ext[p.rows.n - 1] % kRowsPerWave == 0 && p.rows_per_block % (rpw * kRowsPerWave) == 0 &&
                       (!(p.has_add && p.sy_last == 1 && lacking % rpw == 0) || lacking % (rpw * kRowsPerWave) == 0);   // (never at the price of a shared row)
    p.share_add = vec && p.has_add && p.sy_last == 1 && p.rows.n >= 1 && lacking % (multi ? rpw * kRowsPerWave : rpw) == 0;
    hipStream_t st = (hipStream_t)stream;
    dim3 grid;
    if (!vec) {
        int rc = tuple_grid(p.rows_per_block, 1, p.n_tuples, grid);
        if (rc) return rc;
        EG_LAUNCH(k_softmax_rows_scalar, grid, dim3(kThreads), 0, st, p);
        return check_launch("k_softmax_rows_scalar");
    }
    int rc = tuple_grid(p.rows_per_block, multi ? rpw * kRowsPerWave : rpw, p.n_tuples, grid);
    if (rc) return rc;
    const int vpl = (p.n + 511) / 512;
    if (multi) {
        const int add = !p.has_add ? 0 : p.share_add ? 1 : 2;
#define EG_SMB(V) do { if (add == 0) EG_LAUNCH((k_softmax_rows_bf16<V, kRowsPerWave, 0>), grid, dim3(kThreads), 0, st, p); \
                       else if (add == 1) EG_LAUNCH((k_softmax_rows_bf16<V, kRowsPerWave, 1>), grid, dim3(kThreads), 0, st, p); \
                       else EG_LAUNCH((k_softmax_rows_bf16<V, kRowsPerWave, 2>), grid, dim3(kThreads), 0, st, p); } while (0)
        if (vpl <= 1) EG_SMB(1);
        else if (vpl <= 2) EG_SMB(2);
        else EG_SMB(4);
#undef EG_SMB
        return check_launch("k_softmax_rows_bf16");
    }
    if (p.n_tail > 0) {                                // tails: only with run-time dtypes, rows of up to 2048 elements in registers
        if (vpl <= 1) EG_LAUNCH((k_softmax_rows<1, 2, true>), grid, dim3(kThreads), 0, st, p);
        else if (vpl <= 2) EG_LAUNCH((k_softmax_rows<2, 2, true>), grid, dim3(kThreads), 0, st, p);
        else EG_LAUNCH((k_softmax_rows<4, 2, true>), grid, dim3(kThreads), 0, st, p);
        return check_launch("k_softmax_rows");
    }
    const bool all_bf16 = p.dt_src == EG_BF16 && p.dt_t == EG_BF16 && p.dt_e == EG_BF16 && p.dt_p == EG_BF16;
    const bool all_f32 = p.dt_src == EG_F32 && p.dt_t == EG_F32 && p.dt_e == EG_F32 && p.dt_p == EG_F32;
    const int mode = all_bf16 ? 0 : all_f32 ? 1 : 2;
#define EG_SM(V) do { if (mode == 0) EG_LAUNCH((k_softmax_rows<V, 0, false>), grid, dim3(kThreads), 0, st, p); \
                      else if (mode == 1) EG_LAUNCH((k_softmax_rows<V, 1, false>), grid, dim3(kThreads), 0, st, p); \
                      else EG_LAUNCH((k_softmax_rows<V, 2, false>), grid, dim3(kThreads), 0, st, p); } while (0)
    if (vpl <= 1) EG_SM(1);
    else if (vpl <= 2) EG_SM(2);
    else if (vpl <= 4) EG_SM(4);
    else if (vpl <= 8) EG_SM(8);
    else EG_SM(16);
#undef EG_SM
    return check_launch("k_softmax_rows");
}

}  // namespace eg
