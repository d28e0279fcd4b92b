// Bandwidth-bound kernels: element-wise maps, row reductions, the generic one-output-per-lane EinSum
// and the aggregation of partial slabs.
//
// Paper passages: the unary / element-wise forms of EinSum and the softmax pieces are Section 3; the
// per-block kernel K (the inner EinSum on one pair of sub-tensors) is Section 4.3; the aggregation
// operator (group by the surviving key, reduce with (+)) is Section 4.2.  One launch covers every
// tuple of the join: the workgroup index selects (tuple, piece of that tuple's block).
#include <hip/hip_runtime.h>

#include "eg_device.h"

namespace eg {

constexpr int kThreads = 256;

__device__ __forceinline__ char *out_base(const OutSpec &o, int64_t agg)
{
    // partial mode: slab aggIdx of the fp32 workspace; otherwise the destination tensor itself
    return (char *)o.ptr + (o.slab_elems ? agg * o.slab_elems * 4 : 0);
}

// ------------------------------------------------------------------------------------------------
// generic EinSum: one output element per lane, sequential fp32 loop over the aggregated labels
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
        for (int64_t it = 0; it < outer; it++) {
            int64_t bx = ox, by = oy;
            for (int i = 0; i < last; i++) {
                bx += (int64_t)idx[i] * p.rdims.sx[i];
                by += (int64_t)idx[i] * p.rdims.sy[i];
            }
            for (int32_t r = 0; r < ln; r++) {
                float x = load_elem(p.x, p.dtx, bx + r * lsx);
                float y = p.binary ? load_elem(p.y, p.dty, by + r * lsy) : 0.f;
                acc = oplus_eval(p.oplus, acc, otimes_eval(p.otimes, x, y, p.alpha));
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
// element-wise map / binary join without aggregated labels; VEC elements per lane along the last dim
// ------------------------------------------------------------------------------------------------
template <int VEC>
__global__ __launch_bounds__(kThreads) void k_map(const MapParams p)
{
    const int64_t gid = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (gid >= p.n_tuples * p.vecs_per_block) return;
    const int64_t t = gid / p.vecs_per_block;
    int64_t e = gid - t * p.vecs_per_block;
    int64_t ox, oy, oz, agg;
    decode_tuple(p.ts, t, ox, oy, oz, agg);
    const int vd = p.dims.n - 1;
    {   // last dim advances in steps of VEC, the others element by element
        const int64_t nv = (p.dims.ext[vd] + VEC - 1) / VEC;
        int64_t q = e / nv, k = (e - q * nv) * VEC;
        e = q;
        ox += k * p.dims.sx[vd]; oy += k * p.dims.sy[vd]; oz += k * p.dims.sz[vd];
        for (int i = vd - 1; i >= 0; i--) {
            int64_t q2 = e / p.dims.ext[i], k2 = e - q2 * p.dims.ext[i];
            e = q2;
            ox += k2 * p.dims.sx[i]; oy += k2 * p.dims.sy[i]; oz += k2 * p.dims.sz[i];
        }
    }
    char *zb = out_base(p.out, agg);
    if (VEC == 8) {
        float x[8], y[8], z[8];
        if (p.dims.sx[vd] == 1) load8(p.x, p.dtx, ox, x);
        else { float s = load_elem(p.x, p.dtx, ox);
#pragma unroll
            for (int i = 0; i < 8; i++) x[i] = s; }
        if (p.binary) {
            if (p.dims.sy[vd] == 1) load8(p.y, p.dty, oy, y);
            else { float s = load_elem(p.y, p.dty, oy);
#pragma unroll
                for (int i = 0; i < 8; i++) y[i] = s; }
        } else {
#pragma unroll
            for (int i = 0; i < 8; i++) y[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < 8; i++) z[i] = otimes_eval(p.otimes, x[i], y[i], p.alpha);
        store8(zb, p.out.dtype, oz, z);
    } else {
        float x = load_elem(p.x, p.dtx, ox);
        float y = p.binary ? load_elem(p.y, p.dty, oy) : 0.f;
        store_elem(zb, p.out.dtype, oz, otimes_eval(p.otimes, x, y, p.alpha));
    }
}

// ------------------------------------------------------------------------------------------------
// row reduction: LANES lanes cooperate on one output element; the reduced labels are X's trailing dims
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_reduce(int oplus, float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = oplus_eval(oplus, v, __shfl_xor(v, off, 64));
    return v;
}

template <int LANES, int VEC>
__global__ __launch_bounds__(kThreads) void k_reduce_row(const ReduceParams p)
{
    constexpr int PER_WG = kThreads / LANES;
    __shared__ float red[kThreads / 64];
    const int sub = threadIdx.x / LANES, lane = threadIdx.x % LANES;
    const int64_t o = (int64_t)blockIdx.x * PER_WG + sub;
    const bool active = o < p.n_tuples * p.outs_per_block;     // whole lane groups are active or not
    float acc = oplus_identity(p.oplus);
    int64_t oz = 0, agg = 0;
    if (active) {
        const int64_t t = o / p.outs_per_block, e = o - t * p.outs_per_block;
        int64_t ox, oy;
        decode_tuple(p.ts, t, ox, oy, oz, agg);
        decode_dims(p.zdims, e, ox, oy, oz);
        const int vd = p.rdims.n - 1;
        const int64_t nv = (p.rdims.ext[vd] + VEC - 1) / VEC;
        const int64_t total = (p.red_elems / p.rdims.ext[vd]) * nv;
        for (int64_t j = lane; j < total; j += LANES) {
            int64_t q = j / nv, k = (j - q * nv) * VEC;
            int64_t bx = ox + k * p.rdims.sx[vd], by = oy + k * p.rdims.sy[vd];
            for (int i = vd - 1; i >= 0; i--) {
                int64_t q2 = q / p.rdims.ext[i], k2 = q - q2 * p.rdims.ext[i];
                q = q2;
                bx += k2 * p.rdims.sx[i]; by += k2 * p.rdims.sy[i];
            }
            if (VEC == 8) {
                float x[8], y[8];
                load8(p.x, p.dtx, bx, x);
                if (p.binary) {
                    if (p.rdims.sy[vd] == 1) load8(p.y, p.dty, by, y);
                    else { float s = load_elem(p.y, p.dty, by);
#pragma unroll
                        for (int i = 0; i < 8; i++) y[i] = s; }
                } else {
#pragma unroll
                    for (int i = 0; i < 8; i++) y[i] = 0.f;
                }
#pragma unroll
                for (int i = 0; i < 8; i++) acc = oplus_eval(p.oplus, acc, otimes_eval(p.otimes, x[i], y[i], p.alpha));
            } else {
                float x = load_elem(p.x, p.dtx, bx);
                float y = p.binary ? load_elem(p.y, p.dty, by) : 0.f;
                acc = oplus_eval(p.oplus, acc, otimes_eval(p.otimes, x, y, p.alpha));
            }
        }
    }
    acc = wave_reduce(p.oplus, acc);
    if (LANES > 64) {                       // one output per workgroup: combine the four waves through LDS
        if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            float v = red[0];
            for (int w = 1; w < kThreads / 64; w++) v = oplus_eval(p.oplus, v, red[w]);
            if (active) store_elem(out_base(p.out, agg), p.out.dtype, oz, v);
        }
    } else if (lane == 0 && active) {
        store_elem(out_base(p.out, agg), p.out.dtype, oz, acc);
    }
}

// ------------------------------------------------------------------------------------------------
// aggregation of partial slabs: out[e] = (+)_{a ascending} partials[a][e], fp32, one final cast
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads) void k_aggregate_vec4(const AggregateParams p)
{
    const int64_t i4 = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    const int64_t e = i4 * 4;
    if (e >= p.slab_elems) return;
    const float4 *src = (const float4 *)(p.partials + e);
    const int64_t slab4 = p.slab_elems / 4;
    float4 acc = src[0];
    if (p.oplus == EG_AGG_MAX) {
#pragma unroll 4
        for (int64_t a = 1; a < p.n_agg; a++) {
            float4 v = src[a * slab4];
            acc.x = fmaxf(acc.x, v.x); acc.y = fmaxf(acc.y, v.y); acc.z = fmaxf(acc.z, v.z); acc.w = fmaxf(acc.w, v.w);
        }
    } else {
#pragma unroll 4
        for (int64_t a = 1; a < p.n_agg; a++) {
            float4 v = src[a * slab4];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    if (p.out_dtype == EG_BF16) {
        uint2 r;
        r.x = (uint32_t)f32_to_bf16(acc.x) | ((uint32_t)f32_to_bf16(acc.y) << 16);
        r.y = (uint32_t)f32_to_bf16(acc.z) | ((uint32_t)f32_to_bf16(acc.w) << 16);
        *(uint2 *)((uint16_t *)p.out + e) = r;
    } else {
        *(float4 *)((float *)p.out + e) = acc;
    }
}

__global__ __launch_bounds__(kThreads) void k_aggregate_scalar(const AggregateParams p)
{
    const int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (e >= p.slab_elems) return;
    float acc = p.partials[e];
    for (int64_t a = 1; a < p.n_agg; a++) acc = oplus_eval(p.oplus, acc, p.partials[a * p.slab_elems + e]);
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
    hipLaunchKernelGGL(k_generic, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return check_launch("k_generic");
}

int launch_map(const MapParams &p, void *stream)
{
    if (!p.x || (p.binary && !p.y) || !p.out.ptr) return fail(EG_ERR_NULL, "map kernel: NULL operand");
    if (p.dims.n < 1) return fail(EG_ERR_LIMIT, "map kernel: empty index space");
    if (p.vec != 1 && p.vec != 8) return fail(EG_ERR_LIMIT, "map kernel: vector width %d", p.vec);
    unsigned grid;
    int rc = grid_for(p.n_tuples * p.vecs_per_block, kThreads, grid);
    if (rc) return rc;
    if (p.vec == 8) hipLaunchKernelGGL(k_map<8>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    else hipLaunchKernelGGL(k_map<1>, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return check_launch("k_map");
}

int launch_reduce_row(const ReduceParams &p, void *stream)
{
    if (!p.x || (p.binary && !p.y) || !p.out.ptr) return fail(EG_ERR_NULL, "reduce kernel: NULL operand");
    if (p.rdims.n < 1) return fail(EG_ERR_LIMIT, "reduce kernel: empty reduction space");
    const int64_t outs = p.n_tuples * p.outs_per_block;
    const bool wide = p.red_elems >= 16384 || outs < 1024;     // long rows or few rows: a workgroup per output
    unsigned grid;
    int rc = grid_for(outs, wide ? 1 : kThreads / 64, grid);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (wide) {
        if (p.vec == 8) hipLaunchKernelGGL((k_reduce_row<256, 8>), dim3(grid), dim3(kThreads), 0, st, p);
        else hipLaunchKernelGGL((k_reduce_row<256, 1>), dim3(grid), dim3(kThreads), 0, st, p);
    } else {
        if (p.vec == 8) hipLaunchKernelGGL((k_reduce_row<64, 8>), dim3(grid), dim3(kThreads), 0, st, p);
        else hipLaunchKernelGGL((k_reduce_row<64, 1>), dim3(grid), dim3(kThreads), 0, st, p);
    }
    return check_launch("k_reduce_row");
}

int launch_aggregate(const AggregateParams &p, void *stream)
{
    if (!p.partials || !p.out) return fail(EG_ERR_NULL, "aggregate kernel: NULL operand");
    if (p.n_agg < 1 || p.slab_elems < 1) return fail(EG_ERR_LIMIT, "aggregate kernel: empty input");
    const bool vec = p.contiguous && p.slab_elems % 4 == 0 && ((uintptr_t)p.partials & 15) == 0 &&
                     ((uintptr_t)p.out & 15) == 0;
    unsigned grid;
    int rc = grid_for(vec ? p.slab_elems / 4 : p.slab_elems, kThreads, grid);
    if (rc) return rc;
    if (vec) hipLaunchKernelGGL(k_aggregate_vec4, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    else hipLaunchKernelGGL(k_aggregate_scalar, dim3(grid), dim3(kThreads), 0, (hipStream_t)stream, p);
    return check_launch("k_aggregate");
}

}  // namespace eg
