// Executor: routes every annotated vertex to a kernel family, lays out the workspace and launches
// join kernel + aggregation per vertex in topological order.
//
// Paper passages: a vertex runs as a join followed by an aggregation, with an optional repartition
// between vertices when the producer's output partitioning differs from the consumer's input
// partitioning (Section 5); the two-step form temp <- join, res <- aggregation is the end of Section
// 4.3.  Blocks are strided views of dense buffers here, so a repartition rewrites tables only.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <map>
#include <mutex>

#include "eg_internal.h"

namespace eg {

static inline int64_t dtype_size(int dt) { return dt == EG_BF16 ? 2 : 4; }
static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }

struct Operand {
    const void *ptr = nullptr;
    int dtype = EG_F32;
    std::vector<int64_t> stride;     // per dimension of the tensor
};

static std::vector<int64_t> dense_strides(const std::vector<int64_t> &bound)
{
    std::vector<int64_t> st(bound.size());
    int64_t acc = 1;
    for (int i = (int)bound.size() - 1; i >= 0; i--) {
        st[i] = acc;
        acc *= bound[i];
    }
    return st;
}

static int64_t numel(const std::vector<int64_t> &bound)
{
    int64_t n = 1;
    for (int64_t b : bound) n *= b;
    return n;
}

// Per schema label: stride in each operand (0 when the label is absent), block extent.
struct LabelInfo {
    int nl = 0;
    int64_t sx[kMaxLabels] = {0}, sy[kMaxLabels] = {0}, sz[kMaxLabels] = {0};
    bool inx[kMaxLabels] = {false}, iny[kMaxLabels] = {false}, inz[kMaxLabels] = {false};
    int64_t ext[kMaxLabels] = {0};
};

static LabelInfo label_info(const Vertex &v, const Operand &X, const Operand *Y, const std::vector<int64_t> &zstride)
{
    LabelInfo li;
    li.nl = (int)v.labels.size();
    for (int l = 0; l < li.nl; l++) li.ext[l] = v.lbound[l] / v.d[l];
    for (size_t i = 0; i < v.lx.size(); i++) { li.sx[v.lx[i]] = X.stride[i]; li.inx[v.lx[i]] = true; }
    if (Y)
        for (size_t i = 0; i < v.ly.size(); i++) { li.sy[v.ly[i]] = Y->stride[i]; li.iny[v.ly[i]] = true; }
    for (size_t i = 0; i < v.lz.size(); i++) { li.sz[v.lz[i]] = zstride[i]; li.inz[v.lz[i]] = true; }
    return li;
}

// Only partitioned labels (d > 1) enter the device-side tuple space: the others have key 0 in every tuple,
// and the kernels pay scalar instructions per entry.  Row-major order over the kept labels is unchanged.
static TupleSpace tuple_space(const Vertex &v, const LabelInfo &li)
{
    TupleSpace ts;
    memset(&ts, 0, sizeof ts);
    int32_t aggw[kMaxLabels] = {0};
    int64_t w = 1;
    for (int i = (int)v.agg.size() - 1; i >= 0; i--) {
        aggw[v.agg[i]] = (int32_t)w;
        w *= v.d[v.agg[i]];
    }
    int32_t grpw[kMaxLabels] = {0};
    w = 1;
    for (int l = li.nl - 1; l >= 0; l--) {
        if (v.d[l] <= 1 || aggw[l] > 0) continue;
        grpw[l] = (int32_t)w;
        w *= v.d[l];
    }
    int n = 0;
    for (int l = 0; l < li.nl; l++) {
        if (v.d[l] <= 1) continue;
        ts.d[n] = v.d[l];
        ts.step_x[n] = li.ext[l] * li.sx[l];
        ts.step_y[n] = li.ext[l] * li.sy[l];
        ts.step_z[n] = li.ext[l] * li.sz[l];
        ts.agg_w[n] = aggw[l];
        ts.grp_w[n] = grpw[l];
        n++;
    }
    ts.n = n;
    return ts;
}

// Builds a collapsed index space from schema labels (outermost first): extent-1 labels are dropped and
// neighbours are fused when, in every operand, the outer stride equals inner stride * inner extent.
static bool collapse(const LabelInfo &li, const std::vector<int> &labs, StridedDims &out)
{
    memset(&out, 0, sizeof out);
    struct D { int64_t e, x, y, z; };
    std::vector<D> ds;
    for (int l : labs)
        if (li.ext[l] > 1) ds.push_back({li.ext[l], li.sx[l], li.sy[l], li.sz[l]});
    std::vector<D> m;
    for (const D &c : ds) {
        if (!m.empty()) {
            D &p = m.back();
            if (p.x == c.x * c.e && p.y == c.y * c.e && p.z == c.z * c.e && p.e * c.e < (1ll << 31)) {
                p.e *= c.e; p.x = c.x; p.y = c.y; p.z = c.z;
                continue;
            }
        }
        m.push_back(c);
    }
    if ((int)m.size() > kMaxDims) return false;
    out.n = (int)m.size();
    for (int i = 0; i < out.n; i++) {
        if (m[i].e >= (1ll << 31)) return false;
        out.ext[i] = (int32_t)m[i].e; out.sx[i] = m[i].x; out.sy[i] = m[i].y; out.sz[i] = m[i].z;
    }
    return true;
}

static bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }

// Can an operand be read with 16-byte vectors along collapsed dim `vd` of `dims`?  which: 0 = X, 1 = Y.
static bool vec_ok(const StridedDims &dims, int which, int vd, int vec, const void *ptr, const TupleSpace &ts, bool allow_bcast)
{
    const int64_t *s = which == 0 ? dims.sx : dims.sy;
    if (!aligned16(ptr)) return false;
    if (s[vd] == 0) return allow_bcast;
    if (s[vd] != 1) return false;
    for (int i = 0; i < dims.n; i++)
        if (i != vd && s[i] % vec) return false;
    const int64_t *step = which == 0 ? ts.step_x : ts.step_y;
    for (int l = 0; l < ts.n; l++)
        if (step[l] % vec) return false;
    return true;
}

// ------------------------------------------------------------------------------------------------
// contraction eligibility and parameter construction
// ------------------------------------------------------------------------------------------------
static bool build_contract(const Vertex &v, const LabelInfo &li, const Operand &X, const Operand &Y, ContractParams &cp)
{
    if (v.n_in != 2 || (v.oplus != EG_AGG_SUM && v.oplus != EG_AGG_MAX)) return false;
    if (X.dtype != Y.dtype) return false;
    const int epc = X.dtype == EG_BF16 ? 8 : 4;
    if (!aligned16(X.ptr) || !aligned16(Y.ptr)) return false;
    std::vector<int> gb, gm, gn, gk;
    for (int l = 0; l < li.nl; l++) {
        const bool x = li.inx[l], y = li.iny[l], z = li.inz[l];
        if (x && y && z) gb.push_back(l);
        else if (x && z) gm.push_back(l);
        else if (y && z) gn.push_back(l);
        else if (x && y) gk.push_back(l);
        else return false;                     // a label summed out of one operand alone: not a matrix product
    }
    auto live = [&](std::vector<int> &g) { g.erase(std::remove_if(g.begin(), g.end(), [&](int l) { return li.ext[l] <= 1; }), g.end()); };
    live(gb); live(gm); live(gn); live(gk);
    if (gm.empty() || gn.empty() || gk.empty()) return false;
    // the label each operand is contiguous along (stride 1, extent > 1)
    int cx = -1, cy = -1;
    for (int l = 0; l < li.nl; l++) {
        if (li.inx[l] && li.ext[l] > 1 && li.sx[l] == 1) cx = l;
        if (li.iny[l] && li.ext[l] > 1 && li.sy[l] == 1) cy = l;
    }
    if (cx < 0 || cy < 0) return false;
    auto in = [](const std::vector<int> &g, int l) { return std::find(g.begin(), g.end(), l) != g.end(); };
    const bool a_k = in(gk, cx), a_m = in(gm, cx);
    const bool b_k = in(gk, cy), b_n = in(gn, cy);
    if (!(a_k || a_m) || !(b_k || b_n)) return false;
    if (a_k && b_k && cx != cy) return false;
    if (li.ext[cx] % epc || li.ext[cy] % epc) return false;
    for (int l = 0; l < li.nl; l++) {
        if (li.inx[l] && l != cx && li.ext[l] > 1 && li.sx[l] % epc) return false;
        if (li.iny[l] && l != cy && li.ext[l] > 1 && li.sy[l] % epc) return false;
        if ((li.ext[l] * li.sx[l]) % epc || (li.ext[l] * li.sy[l]) % epc) return false;   // block steps keep alignment
    }
    // order each group outermost-first by stride in its leading operand, contiguous label last
    auto order = [&](std::vector<int> &g, const int64_t *s, int last) {
        std::sort(g.begin(), g.end(), [&](int a, int b) { return s[a] > s[b]; });
        if (last >= 0 && in(g, last)) {
            g.erase(std::find(g.begin(), g.end(), last));
            g.push_back(last);
        }
    };
    order(gb, li.sx, -1);
    order(gm, li.sx, a_m ? cx : -1);
    order(gn, li.sy, b_n ? cy : -1);
    order(gk, li.sx, a_k ? cx : (b_k ? cy : -1));
    // fuse neighbours where every operand that carries the group allows it
    auto fill = [&](const std::vector<int> &g, DimList &dl, const int64_t *s0, const int64_t *s1, const int64_t *s2) -> bool {
        struct D { int64_t e, a, b, c; };
        std::vector<D> m;
        for (int l : g) {
            D c{li.ext[l], s0 ? s0[l] : 0, s1 ? s1[l] : 0, s2 ? s2[l] : 0};
            if (!m.empty()) {
                D &p = m.back();
                if (p.a == c.a * c.e && p.b == c.b * c.e && p.c == c.c * c.e && p.e * c.e < (1ll << 31)) {
                    p.e *= c.e; p.a = c.a; p.b = c.b; p.c = c.c;
                    continue;
                }
            }
            m.push_back(c);
        }
        if ((int)m.size() > kMaxGroup) return false;
        memset(&dl, 0, sizeof dl);
        dl.n = (int)m.size();
        for (int i = 0; i < dl.n; i++) {
            if (m[i].e >= (1ll << 31)) return false;
            dl.ext[i] = (int32_t)m[i].e; dl.s0[i] = m[i].a; dl.s1[i] = m[i].b; dl.s2[i] = m[i].c;
        }
        return true;
    };
    memset(&cp, 0, sizeof cp);
    if (!fill(gb, cp.batch, li.sx, li.sy, li.sz)) return false;
    if (!fill(gm, cp.m, li.sx, li.sz, nullptr)) return false;
    if (!fill(gn, cp.n, li.sy, li.sz, nullptr)) return false;
    if (!fill(gk, cp.k, li.sx, li.sy, nullptr)) return false;
    auto size = [](const DimList &d) { int64_t p = 1; for (int i = 0; i < d.n; i++) p *= d.ext[i]; return p; };
    cp.M = size(cp.m); cp.N = size(cp.n); cp.K = size(cp.k); cp.n_batch = size(cp.batch);
    if (cp.M >= (1ll << 31) || cp.N >= (1ll << 31) || cp.K >= (1ll << 31)) return false;
    cp.a_kcontig = a_k ? 1 : 0;
    cp.b_kcontig = b_k ? 1 : 0;
    // after fusing, the innermost entry of the vectorised group must still be the stride-1 run
    if (a_k && cp.k.s0[cp.k.n - 1] != 1) return false;
    if (!a_k && cp.m.s0[cp.m.n - 1] != 1) return false;
    if (b_k && cp.k.s1[cp.k.n - 1] != 1) return false;
    if (!b_k && cp.n.s0[cp.n.n - 1] != 1) return false;
    if (a_k && cp.k.ext[cp.k.n - 1] % epc) return false;
    if (!a_k && cp.m.ext[cp.m.n - 1] % epc) return false;
    if (b_k && cp.k.ext[cp.k.n - 1] % epc) return false;
    if (!b_k && cp.n.ext[cp.n.n - 1] % epc) return false;
    for (int l = 0; l < li.nl; l++) {
        cp.span_x += (li.ext[l] - 1) * li.sx[l];
        cp.span_y += (li.ext[l] - 1) * li.sy[l];
    }
    cp.in_dtype = X.dtype;
    cp.otimes = v.otimes;
    cp.oplus = v.oplus;
    cp.alpha = (float)v.alpha;
    cp.x = X.ptr;
    cp.y = Y.ptr;
    return true;
}

// ------------------------------------------------------------------------------------------------
// routing of one vertex given the real strides of its operands
// ------------------------------------------------------------------------------------------------
struct Routed {
    int kind = EG_KERNEL_NONE;
    bool swapped = false;          // contraction: X and Y changed places (see route)
    ContractParams cp;
    MapParams mp;
    ReduceParams rp;
    GenericParams gp;
};

// How many pieces the reduction range of every output is cut into when a row reduction has too few
// outputs to fill the chip: each piece becomes one more partial slab for the aggregation kernel.
static int reduce_split(int64_t outs_total, int64_t red_elems)
{
    if (outs_total >= 1024 || red_elems < 32768) return 1;
    int64_t s = (1024 + outs_total - 1) / outs_total;
    if (s > red_elems / 8192) s = red_elems / 8192;
    return s < 1 ? 1 : (int)s;                      // at most 1024 pieces of at least 8192 elements
}

// The same for a column reduction.  There a lane owns a vector of 8 outputs and keeps four 16-byte loads in flight,
// and 8 lane groups of a workgroup share a piece: enough pieces for some 512 K lanes (64 bytes each, which is what
// the memory system needs in flight: 128 K lanes reached 3.0 TB/s, 512 K 5.3), each lane with at least 16 steps.
static int column_split(int64_t vectors_total, int64_t red_elems)
{
    const int64_t lanes = vectors_total * 8;
    if (lanes >= 524288 || red_elems < 256) return 1;
    int64_t s = (524288 + lanes - 1) / lanes;
    if (s > red_elems / 128) s = red_elems / 128;
    if (s > 64) s = 64;
    return s < 1 ? 1 : (int)s;
}

// split: 0 = decide here (dry run), otherwise the value fixed when the workspace was laid out
static int route(const Vertex &v, const Operand &X, const Operand *Y, const std::vector<int64_t> &zstride,
                 const OutSpec &out, Routed &r, int split = 0)
{
    LabelInfo li = label_info(v, X, Y, zstride);
    TupleSpace ts = tuple_space(v, li);
    const int64_t n_tuples = v.plan.n_tuples;
    const bool binary = v.n_in == 2;

    if (v.agg.empty()) {                                        // element-wise: no aggregated label
        auto build = [&](const LabelInfo &li, const TupleSpace &ts, int64_t n_tuples) -> bool {
            MapParams &p = r.mp;
            memset(&p, 0, sizeof p);
            std::vector<int> zl(v.lz.begin(), v.lz.end());
            if (!collapse(li, zl, p.dims)) return false;
            if (p.dims.n == 0) { p.dims.n = 1; p.dims.ext[0] = 1; }
            p.ts = ts; p.binary = binary; p.otimes = v.otimes; p.alpha = (float)v.alpha;
            p.dtx = X.dtype; p.dty = Y ? Y->dtype : EG_F32;
            p.x = X.ptr; p.y = Y ? Y->ptr : nullptr; p.out = out; p.n_tuples = n_tuples;
            const int vd = p.dims.n - 1;
            // whole 16-byte vectors, except in a dense one-dimensional space that is not cut: there the last vector may be partial
            const bool flat = p.dims.n == 1 && ts.n == 0;
            bool vz = p.dims.sz[vd] == 1 && aligned16(out.ptr) && (p.dims.ext[vd] % 8 == 0 || flat);
            for (int i = 0; i < p.dims.n && vz; i++)
                if (i != vd && p.dims.sz[i] % 8) vz = false;
            for (int l = 0; l < ts.n && vz; l++)
                if (ts.step_z[l] % 8) vz = false;
            if (out.slab_elems % 8) vz = false;
            bool vx = vec_ok(p.dims, 0, vd, 8, X.ptr, ts, true);
            bool vy = !binary || vec_ok(p.dims, 1, vd, 8, Y->ptr, ts, true);
            p.vec = (vz && vx && vy) ? 8 : 1;
            // one operand contiguous along another dimension than Z's last (a transpose): tiles through LDS
            if (p.vec == 1 && vz && p.dims.n >= 2 && (!binary || vx != vy) && (binary || !vx)) {
                const bool xt = !vx;
                const int64_t *s = xt ? p.dims.sx : p.dims.sy;
                const int64_t *step = xt ? ts.step_x : ts.step_y;
                int td = -1;
                for (int i = 0; i < vd; i++)
                    if (s[i] == 1 && p.dims.ext[i] % 8 == 0) td = i;
                bool ok = td >= 0 && aligned16(xt ? X.ptr : Y->ptr);
                for (int i = 0; i < p.dims.n && ok; i++)
                    if (i != td && s[i] % 8) ok = false;
                for (int l = 0; l < ts.n && ok; l++)
                    if (step[l] % 8) ok = false;
                if (ok) { p.tr = xt ? 1 : 2; p.td = td; p.vec = 8; }
            }
            int64_t rows = 1;
            for (int i = 0; i < vd; i++) rows *= p.dims.ext[i];
            p.vecs_per_block = rows * ((p.dims.ext[vd] + p.vec - 1) / p.vec);
            return true;
        };
        // A scalar function applied block by block is the same function applied to the whole tensors, and the blocks of
        // every operand under one key lie where the whole tensor has them, so the tuples are walked as one index space
        // in memory order (a tensor cut eight ways along its rows or inside them streams like an uncut one); the tuple
        // by tuple launch remains for spaces too large for one and for those without 16-byte accesses.
        if (ts.n > 0) {
            LabelInfo whole = li;
            for (int l = 0; l < li.nl; l++) whole.ext[l] = v.lbound[l];
            TupleSpace none;
            memset(&none, 0, sizeof none);
            if (build(whole, none, 1) && r.mp.vec == 8 && r.mp.vecs_per_block < (1ll << 32)) { r.kind = EG_KERNEL_MAP; return EG_OK; }
        }
        if (!build(li, ts, n_tuples)) return fail(EG_ERR_LIMIT, "map: too many dimensions after collapsing");
        r.kind = EG_KERNEL_MAP;
        return EG_OK;
    }

    // Z contiguous along a label that only X carries: with a symmetric scalar function the operands change places,
    // so that label becomes a column label and result tiles are written along their rows in 16-byte vectors
    // (same products, same order of summation; `ij,jk->ki` ran 30 % slower than `ij,jk->ik` before).
    bool swap = false;
    if (binary && (v.otimes == EG_MUL || v.otimes == EG_SQDIFF || v.otimes == EG_ABSDIFF))   // not ADD: that is alpha * x + y
        for (int l = 0; l < li.nl; l++)
            if (li.inz[l] && li.ext[l] > 1 && li.sz[l] == 1 && li.inx[l] && !li.iny[l]) swap = true;
    LabelInfo lc = li;
    TupleSpace tc = ts;
    if (swap) {
        for (int l = 0; l < li.nl; l++) { std::swap(lc.inx[l], lc.iny[l]); std::swap(lc.sx[l], lc.sy[l]); }
        for (int l = 0; l < ts.n; l++) std::swap(tc.step_x[l], tc.step_y[l]);
    }
    if (binary && build_contract(v, lc, swap ? *Y : X, swap ? X : *Y, r.cp)) {
        r.cp.ts = tc;
        r.cp.out = out;
        r.cp.n_tuples = n_tuples;
        r.swapped = swap;
        r.kind = v.otimes == EG_MUL && v.oplus == EG_AGG_SUM ? EG_KERNEL_CONTRACT_MFMA : EG_KERNEL_CONTRACT_ALU;
        return EG_OK;
    }

    // output and reduction index spaces
    std::vector<int> zl(v.lz.begin(), v.lz.end());
    // row reduction: the aggregated labels are the trailing dimensions of X, and Y has no label outside X
    bool tail = v.lx.size() >= v.agg.size();
    std::vector<int> rl;
    if (tail) {
        for (size_t i = v.lx.size() - v.agg.size(); i < v.lx.size(); i++) {
            if (li.inz[v.lx[i]]) tail = false;
            rl.push_back(v.lx[i]);
        }
        for (int a : v.agg)
            if (!li.inx[a]) tail = false;
    }
    if (tail) {                                  // short reductions are better served one lane per output
        int64_t red = 1;
        for (int a : v.agg) red *= li.ext[a];
        if (red < 64) tail = false;
    }
    bool have_row = false;
    ReduceParams row;
    if (tail) {
        ReduceParams &p = r.rp;
        memset(&p, 0, sizeof p);
        if (collapse(li, zl, p.zdims) && collapse(li, rl, p.rdims)) {
            if (p.rdims.n == 0) { p.rdims.n = 1; p.rdims.ext[0] = 1; }
            p.ts = ts; p.binary = binary; p.otimes = v.otimes; p.oplus = v.oplus; p.alpha = (float)v.alpha;
            p.dtx = X.dtype; p.dty = Y ? Y->dtype : EG_F32;
            p.x = X.ptr; p.y = Y ? Y->ptr : nullptr; p.out = out; p.n_tuples = n_tuples;
            p.outs_per_block = 1;
            for (int i = 0; i < p.zdims.n; i++) p.outs_per_block *= p.zdims.ext[i];
            p.red_elems = 1;
            for (int i = 0; i < p.rdims.n; i++) p.red_elems *= p.rdims.ext[i];
            const int vd = p.rdims.n - 1;
            bool vx = p.rdims.ext[vd] % 8 == 0 && vec_ok(p.rdims, 0, vd, 8, X.ptr, ts, false);
            bool vy = !binary || vec_ok(p.rdims, 1, vd, 8, Y->ptr, ts, true);
            // the output index also moves the vector start: its strides must keep 16-byte alignment
            for (int i = 0; i < p.zdims.n; i++) {
                if (p.zdims.sx[i] % 8) vx = false;
                if (binary && p.zdims.sy[i] % 8) vy = false;
            }
            p.vec = (vx && vy) ? 8 : 1;
            p.split = split > 0 ? split : reduce_split(p.outs_per_block * n_tuples, p.red_elems);
            r.kind = EG_KERNEL_REDUCE_ROW;
            if (p.vec == 8) return EG_OK;
            have_row = true;                    // element by element: only if the column form below does not apply
            row = p;
        }
    }

    // column reduction: the outputs' innermost dimension is contiguous in X and in Z, so lanes can own vectors of
    // outputs; the aggregated labels lie anywhere else in X
    {
        ReduceParams &p = r.rp;
        memset(&p, 0, sizeof p);
        std::vector<int> al(v.agg.begin(), v.agg.end());
        bool ok = true;
        for (int a : v.agg)
            if (!li.inx[a]) ok = false;
        if (ok && collapse(li, zl, p.zdims) && collapse(li, al, p.rdims) && p.zdims.n >= 1 && p.rdims.n >= 1) {
            const int zd = p.zdims.n - 1;
            p.outs_per_block = 1;
            for (int i = 0; i < p.zdims.n; i++) p.outs_per_block *= p.zdims.ext[i];
            p.red_elems = 1;
            for (int i = 0; i < p.rdims.n; i++) p.red_elems *= p.rdims.ext[i];
            // along that dimension an operand is read in 16-byte vectors (stride 1) or as one value (stride 0, or absent)
            const bool xvec = p.zdims.sx[zd] == 1, yvec = binary && p.zdims.sy[zd] == 1;
            ok = p.zdims.ext[zd] % 8 == 0 && p.zdims.sz[zd] == 1 && aligned16(out.ptr) && out.slab_elems % 8 == 0 &&
                 p.red_elems >= 16 && p.red_elems < (1ll << 32) && (xvec || yvec) &&
                 (xvec ? aligned16(X.ptr) : p.zdims.sx[zd] == 0) && (!binary || (yvec ? aligned16(Y->ptr) : p.zdims.sy[zd] == 0));
            for (int i = 0; i < p.zdims.n && ok; i++)
                if (i != zd && ((xvec && p.zdims.sx[i] % 8) || p.zdims.sz[i] % 8 || (yvec && p.zdims.sy[i] % 8))) ok = false;
            for (int i = 0; i < p.rdims.n && ok; i++)
                if ((xvec && p.rdims.sx[i] % 8) || (yvec && p.rdims.sy[i] % 8)) ok = false;
            for (int l = 0; l < ts.n && ok; l++)
                if ((xvec && ts.step_x[l] % 8) || ts.step_z[l] % 8 || (yvec && ts.step_y[l] % 8)) ok = false;
            if (ok) {
                p.ts = ts; p.binary = binary; p.otimes = v.otimes; p.oplus = v.oplus; p.alpha = (float)v.alpha;
                p.dtx = X.dtype; p.dty = Y ? Y->dtype : EG_F32;
                p.x = X.ptr; p.y = Y ? Y->ptr : nullptr; p.out = out; p.n_tuples = n_tuples;
                p.vec = 8;
                p.col = 1;
                p.split = split > 0 ? split : column_split(p.outs_per_block / 8 * n_tuples, p.red_elems);
                r.kind = EG_KERNEL_REDUCE_ROW;
                return EG_OK;
            }
        }
    }

    if (have_row) {
        r.rp = row;
        r.kind = EG_KERNEL_REDUCE_ROW;
        return EG_OK;
    }

    GenericParams &p = r.gp;
    memset(&p, 0, sizeof p);
    std::vector<int> al(v.agg.begin(), v.agg.end());
    if (!collapse(li, zl, p.zdims) || !collapse(li, al, p.rdims))
        return fail(EG_ERR_LIMIT, "generic: too many dimensions after collapsing");
    p.ts = ts; p.binary = binary; p.otimes = v.otimes; p.oplus = v.oplus; p.alpha = (float)v.alpha;
    p.dtx = X.dtype; p.dty = Y ? Y->dtype : EG_F32;
    p.x = X.ptr; p.y = Y ? Y->ptr : nullptr; p.out = out; p.n_tuples = n_tuples;
    p.outs_per_block = 1;
    for (int i = 0; i < p.zdims.n; i++) p.outs_per_block *= p.zdims.ext[i];
    p.red_elems = 1;
    for (int i = 0; i < p.rdims.n; i++) p.red_elems *= p.rdims.ext[i];
    r.kind = EG_KERNEL_GENERIC;
    return EG_OK;
}

// Element stride between the partial slabs of a vertex in the workspace.  More than two slabs of 1 MiB or more
// are spaced 4 KiB further apart than their dense size: slab sizes are often powers of two, and then every lane
// of the aggregation would pull its n_agg vectors from addresses that fall on the same memory channel and bank
// (measured: 5-8 % slower).
static int64_t slab_stride_of(int64_t dense_elems, int64_t slabs)
{
    return slabs > 2 && dense_elems >= (1 << 18) ? dense_elems + 1024 : dense_elems;
}

// ------------------------------------------------------------------------------------------------
// workspace layout: intermediates and partial slabs, first-fit with reuse after the last consumer
// ------------------------------------------------------------------------------------------------
struct Layout {
    std::vector<int64_t> result_off;    // per vertex: byte offset of its tensor in the workspace (-1: not there)
    std::vector<int64_t> partial_off;   // per vertex: byte offset of its partial slabs (-1: none)
    std::vector<int> split;             // per vertex: extra slabs per aggIdx from a split row reduction or contraction (1: none)
    std::vector<int> split_label;       // contraction: the contracted label that is cut `split` times finer
    std::vector<int64_t> aux_off;       // per vertex: byte offset of a launch's own scratch (the one-pass attention's mask classes; -1: none)
    int64_t total = 0;
};

class Arena {
public:
    int64_t alloc(int64_t bytes)
    {
        bytes = align_up(std::max<int64_t>(bytes, 1), 256);
        for (auto it = free_.begin(); it != free_.end(); ++it) {
            if (it->second >= bytes) {
                int64_t off = it->first, rest = it->second - bytes;
                free_.erase(it);
                if (rest) free_[off + bytes] = rest;
                size_[off] = bytes;
                return off;
            }
        }
        int64_t off = top_;
        // grow from a trailing free block if there is one
        if (!free_.empty()) {
            auto last = std::prev(free_.end());
            if (last->first + last->second == top_) {
                off = last->first;
                free_.erase(last);
            }
        }
        top_ = off + bytes;
        size_[off] = bytes;
        return off;
    }
    void release(int64_t off)
    {
        int64_t bytes = size_[off];
        size_.erase(off);
        auto it = free_.emplace(off, bytes).first;
        auto nx = std::next(it);
        if (nx != free_.end() && it->first + it->second == nx->first) {
            it->second += nx->second;
            free_.erase(nx);
        }
        if (it != free_.begin()) {
            auto pv = std::prev(it);
            if (pv->first + pv->second == it->first) {
                pv->second += it->second;
                free_.erase(it);
            }
        }
    }
    int64_t top() const { return top_; }

private:
    std::map<int64_t, int64_t> free_, size_;
    int64_t top_ = 0;
};

static int dry_route(const eg_graph *g, int vertex, Routed &r);

// ------------------------------------------------------------------------------------------------
// fusion of softmax chains (Section 3 of the paper writes softmax as four EinSums)
// ------------------------------------------------------------------------------------------------
struct FuseGroup {
    int add = -1;              // the alpha * x + y vertex in front of the chain, or -1
    int vmax = -1, vexp = -1, vsum = -1, vdiv = -1;
    int src = -1, addend = -1; // what the chain reads: the source tensor and the added operand (or -1)
    bool emit_max = false, emit_sum = false, emit_div = true;
    // element-wise vertices behind the chain that its pass evaluates as well (see SoftmaxTail): the vertices, their operand
    // slots, whether each is still written, and the tensors of full rank they read from outside the group
    std::vector<int> tails, tail_a, tail_b, ext;
    std::vector<char> tail_row, tail_emit;
    // attention as one pass (tr_set_fused_attention): the contraction that produces the chain's source and the contraction
    // that consumes its result join the group; the pass then stands at the second contraction
    int qk = -1, pv = -1;
    int q = -1, k = -1, v = -1;                 // the tensors it reads besides the added operand
    int lab_s = -1, lab_t = -1, lab_d = -1;     // qk's schema indices of the query, key and contracted label
    int lab_dv = -1;                            // pv's schema index of V's own label (the head dimension of the result)
    int anchor() const { return pv >= 0 ? pv : vdiv; }
    std::vector<int> members() const
    {
        std::vector<int> m;
        for (int u : {qk, add, vmax, vexp, vsum, vdiv, pv})
            if (u >= 0) m.push_back(u);
        m.insert(m.end(), tails.begin(), tails.end());
        return m;
    }
    std::vector<int> reads() const
    {
        std::vector<int> r;
        if (pv >= 0) { r = {q, k}; if (addend >= 0) r.push_back(addend); r.push_back(v); }
        else { r.push_back(src); if (addend >= 0) r.push_back(addend); r.insert(r.end(), ext.begin(), ext.end()); }
        return r;
    }
    std::vector<int> writes() const
    {
        if (pv >= 0) return {pv};
        std::vector<int> w;
        if (emit_div) w.push_back(vdiv);
        if (emit_max) w.push_back(vmax);
        if (emit_sum) w.push_back(vsum);
        for (size_t k = 0; k < tails.size(); k++)
            if (tail_emit[k]) w.push_back(tails[k]);
        return w;
    }
};

static bool is_iota(const std::vector<int> &l, size_t n)
{
    if (l.size() != n) return false;
    for (size_t i = 0; i < n; i++)
        if (l[i] != (int)i) return false;
    return true;
}

// Chains max -> exp(x - max) -> sum -> division over the last label that can run as one pass: same partitioning
// vector on every vertex, the reduced label unpartitioned, rows of at most 8192 elements, and no consumer of the
// exponentials (or of the sum alpha * x + y in front) outside the chain.  Row maxima and sums may have other
// consumers as long as those come after the division in vertex order.  A purely structural test: it does not
// depend on strides, so the workspace layout and the execution agree on it.
static std::vector<FuseGroup> find_fusions(const eg_graph *g)
{
    std::vector<FuseGroup> out;
    if (!g->fuse) return out;
    const int nv = (int)g->v.size();
    std::vector<std::vector<int>> cons(nv);
    for (int i = 0; i < nv; i++)
        for (int k = 0; k < g->v[i].n_in; k++)
            if (k == 0 || g->v[i].in[0] != g->v[i].in[1]) cons[g->v[i].in[k]].push_back(i);
    std::vector<char> taken(nv, 0);
    auto only = [&](int u, std::initializer_list<int> allowed) {
        for (int c : cons[u])
            if (std::find(allowed.begin(), allowed.end(), c) == allowed.end()) return false;
        return true;
    };
    for (int p = 0; p < nv; p++) {
        const Vertex &P = g->v[p];
        if (P.is_input || P.n_in != 2 || P.otimes != EG_DIV || !P.agg.empty()) continue;
        const int e = P.in[0], s = P.in[1];
        if (e == s || g->v[e].is_input || g->v[s].is_input) continue;
        const Vertex &E = g->v[e], &S = g->v[s];
        if (E.n_in != 2 || E.otimes != EG_EXP_SUB || !E.agg.empty() || E.is_output) continue;
        if (S.n_in != 1 || S.in[0] != e || S.otimes != EG_IDENT || S.oplus != EG_AGG_SUM) continue;
        const int t = E.in[0], c = E.in[1];
        if (t == c || g->v[c].is_input) continue;
        const Vertex &C = g->v[c];
        if (C.n_in != 1 || C.in[0] != t || C.otimes != EG_IDENT || C.oplus != EG_AGG_MAX) continue;
        const size_t r = E.lx.size();
        if (r < 1) continue;
        // shapes: full-rank operands are labelled 0..r-1 (first-appearance order), the row statistics lack the last label
        if (!is_iota(E.lx, r) || !is_iota(E.ly, r - 1) || !is_iota(E.lz, r)) continue;
        if (!is_iota(P.lx, r) || !is_iota(P.ly, r - 1) || !is_iota(P.lz, r)) continue;
        if (!is_iota(C.lx, r) || !is_iota(C.lz, r - 1) || !is_iota(S.lx, r) || !is_iota(S.lz, r - 1)) continue;
        // the pass runs under the division's partitioning vector; how the vertices inside the chain were cut does not
        // matter (their tensors are dense, a cut is only a view), but a row must lie inside one block
        if (P.d[r - 1] != 1) continue;
        if (E.lbound[r - 1] > 8192) continue;
        if (!only(e, {s, p})) continue;
        if (taken[e] || taken[s] || taken[c] || taken[p]) continue;
        FuseGroup grp;
        grp.vmax = c; grp.vexp = e; grp.vsum = s; grp.vdiv = p; grp.src = t;
        grp.emit_max = C.is_output || !only(c, {e});
        grp.emit_sum = S.is_output || !only(s, {p});
        bool late = true;                       // whoever else reads the statistics must run after the fused pass
        for (int u : cons[c]) late = late && (u == e || u > p);
        for (int u : cons[s]) late = late && (u == p || u > p);
        if (!late) continue;
        // alpha * x + y in front, when it feeds nothing but the chain
        if (!g->v[t].is_input) {
            const Vertex &T = g->v[t];
            if (T.n_in == 2 && T.otimes == EG_ADD && T.agg.empty() && !T.is_output && T.in[0] != T.in[1] && !taken[t] &&
                is_iota(T.lx, r) && is_iota(T.lz, r) && only(t, {c, e})) {
                grp.add = t;
                grp.src = T.in[0];
                grp.addend = T.in[1];
            }
        }
        for (int u : {grp.add, c, e, s, p})
            if (u >= 0) taken[u] = 1;
        out.push_back(grp);
    }
    // Tails: element-wise vertices after the division whose operands are the chain's own values (the source as the chain sees
    // it, the row maximum, the exponentials, the row sum, the quotient), earlier tails, or tensors of the result's shape that
    // exist before the pass runs.  The pass evaluates them on the spot; the chain's values and the tails that nobody else
    // reads are then never stored.  Structural conditions only.
    for (FuseGroup &f : out) {
        const int p = f.vdiv, tsrc = g->v[f.vexp].in[0];
        const Vertex &P = g->v[p];
        const size_t r = P.lz.size();
        std::vector<int> slot_of(nv, -1), per_row(nv, 0);
        slot_of[tsrc] = 0; slot_of[f.vmax] = 1; slot_of[f.vexp] = 2; slot_of[f.vsum] = 3; slot_of[p] = 4;
        per_row[f.vmax] = per_row[f.vsum] = 1;
        for (int j = p + 1; j < nv && j <= p + 12 && (int)f.tails.size() < kSoftmaxTails; j++) {
            const Vertex &T = g->v[j];
            if (T.is_input || taken[j] || !T.agg.empty() || T.n_in < 1 || T.n_in > 2) continue;
            if (T.n_in == 2 && T.in[0] == T.in[1]) continue;
            switch (T.otimes) {                      // the scalar functions the element-wise kernel knows
            case EG_MUL: case EG_ADD: case EG_SUB: case EG_DIV: case EG_SQDIFF: case EG_ABSDIFF: case EG_EXP_SUB: case EG_RELU_GRAD:
            case EG_SILU_MUL: case EG_IDENT: case EG_SCALE: case EG_RELU: case EG_EXP: case EG_LOG: break;
            default: continue;
            }
            const bool row = is_iota(T.lz, r - 1) && r >= 2;
            if (!row && !is_iota(T.lz, r)) continue;
            bool ok = true, inside = false;
            int sl[2] = {-1, -1};
            std::vector<int> ext = f.ext;
            for (int k = 0; k < T.n_in && ok; k++) {
                const int u = T.in[k];
                const std::vector<int> &lab = k == 0 ? T.lx : T.ly;
                if (slot_of[u] >= 0) {
                    ok = per_row[u] ? is_iota(lab, r - 1) : (!row && is_iota(lab, r));
                    sl[k] = slot_of[u];
                    inside = true;
                } else {
                    // a tensor of the result's shape that exists when the pass runs: a graph input or an earlier vertex outside the group
                    ok = !row && is_iota(lab, r) && (g->v[u].is_input || u < p) && g->v[u].bound == P.bound;
                    for (int m : f.members()) ok = ok && u != m;
                    if (!ok) break;
                    size_t e = std::find(ext.begin(), ext.end(), u) - ext.begin();
                    if (e == ext.size()) ext.push_back(u);
                    ok = (int)ext.size() <= kSoftmaxExt;
                    sl[k] = 5 + (int)e;
                }
            }
            if (!ok || !inside) continue;
            for (size_t l = 0; l < T.lz.size() && ok; l++) ok = T.lbound[l] == P.lbound[l];      // same extents, label by label
            if (!ok) continue;
            slot_of[j] = 8 + (int)f.tails.size();
            per_row[j] = row;
            f.tails.push_back(j); f.tail_a.push_back(sl[0]); f.tail_b.push_back(sl[1]); f.tail_row.push_back(row); f.tail_emit.push_back(1);
            f.ext = ext;
            taken[j] = 1;
        }
        if (f.tails.empty()) continue;
        // alpha * x + y in front once more: with tails that read its sum it may now feed nothing but the group
        if (f.add < 0 && !g->v[tsrc].is_input && !taken[tsrc]) {
            const Vertex &T = g->v[tsrc];
            bool inside = T.n_in == 2 && T.otimes == EG_ADD && T.agg.empty() && !T.is_output && T.in[0] != T.in[1] && is_iota(T.lx, r) && is_iota(T.lz, r);
            const std::vector<int> mem0 = f.members();
            for (int c : cons[tsrc]) inside = inside && std::find(mem0.begin(), mem0.end(), c) != mem0.end();
            for (int e : f.ext) inside = inside && e != T.in[0] && e != T.in[1];
            if (inside) {
                f.add = tsrc; f.src = T.in[0]; f.addend = T.in[1];
                taken[tsrc] = 1;
            }
        }
        // what is still written: whatever somebody outside the group reads, or the caller asked for
        std::vector<int> mem = f.members();
        auto wanted = [&](int u) {
            if (g->v[u].is_output) return true;
            for (int c : cons[u])
                if (std::find(mem.begin(), mem.end(), c) == mem.end()) return true;
            return false;
        };
        f.emit_max = wanted(f.vmax);
        f.emit_sum = wanted(f.vsum);
        f.emit_div = wanted(p);
        for (size_t k = 0; k < f.tails.size(); k++) f.tail_emit[k] = wanted(f.tails[k]);
    }
    if (!g->fuse_attention) return out;
    // Attention (Section 3): scores = a contraction whose result [batch.., s, t] feeds nothing but the chain, and a
    // contraction of the chain's result with V over t.  Structural conditions only, as above.
    for (FuseGroup &f : out) {
        if (f.emit_max || f.emit_sum || !f.tails.empty()) continue;
        const int t1 = f.src, p = f.vdiv;
        if (t1 < 0 || g->v[t1].is_input || taken[t1]) continue;
        const Vertex &T1 = g->v[t1], &P = g->v[p];
        if (T1.n_in != 2 || T1.otimes != EG_MUL || T1.oplus != EG_AGG_SUM || T1.is_output || P.is_output || T1.in[0] == T1.in[1]) continue;
        if (f.add >= 0 ? !only(t1, {f.add}) : !only(t1, {f.vmax, f.vexp})) continue;
        const size_t r = T1.lz.size();
        if (r < 2 || r > 4 || r != g->v[f.vexp].lx.size()) continue;
        // label roles in the first contraction
        const int nl = (int)T1.labels.size();
        std::vector<int> inx(nl, 0), iny(nl, 0), inz(nl, 0);
        for (int l : T1.lx) inx[l] = 1;
        for (int l : T1.ly) iny[l] = 1;
        for (int l : T1.lz) inz[l] = 1;
        int ls = T1.lz[r - 2], lt = T1.lz[r - 1], ld = -1, nk = 0;
        bool ok = inx[ls] && !iny[ls] && iny[lt] && !inx[lt];
        for (int l = 0; l < nl; l++)
            if (inx[l] && iny[l] && !inz[l]) { ld = l; nk++; }
        for (size_t i = 0; i + 2 < r; i++) ok = ok && inx[T1.lz[i]] && iny[T1.lz[i]];          // leading labels: batch
        ok = ok && nk == 1 && T1.lx.size() == r && T1.ly.size() == r && (int)T1.agg.size() == 1;   // X: batch labels, s, d;  Y: batch labels, t, d (any order)
        if (!ok || T1.d[ld] != 1) continue;
        const int64_t D = T1.lbound[ld];
        if (D != 32 && D != 64 && D != 128) continue;
        if (f.addend >= 0) {                    // the added operand may carry the query and key labels only
            const Vertex &A = g->v[f.add];
            bool fits = true;
            for (int l : A.ly) fits = fits && (l == (int)r - 2 || l == (int)r - 1);
            if (!fits) continue;
        }
        // the consumer of the chain's result
        if (cons[p].size() != 1) continue;
        const int o = cons[p][0];
        const Vertex &O = g->v[o];
        if (taken[o] || O.n_in != 2 || O.in[0] != p || O.in[1] == p || O.otimes != EG_MUL || O.oplus != EG_AGG_SUM || O.lx.size() != r) continue;
        const int no = (int)O.labels.size();
        std::vector<int> oy(no, 0), oz(no, 0);
        for (int l : O.ly) oy[l] = 1;
        for (int l : O.lz) oz[l] = 1;
        const int os = O.lx[r - 2], ot = O.lx[r - 1];
        bool ok2 = oy[ot] && !oz[ot] && !oy[os] && oz[os];
        for (size_t i = 0; i + 2 < r; i++) ok2 = ok2 && oy[O.lx[i]] && oz[O.lx[i]];
        int ldv = -1, nn = 0;
        for (int l = 0; l < no; l++)
            if (oy[l] && oz[l] && std::find(O.lx.begin(), O.lx.end(), l) == O.lx.end()) { ldv = l; nn++; }
        ok2 = ok2 && nn == 1 && O.ly.size() == r && O.lz.size() == r && (int)O.agg.size() == 1;
        if (!ok2 || O.d[ot] != 1 || O.lbound[ldv] != D) continue;
        if (g->v[T1.in[0]].dtype != EG_BF16 || g->v[T1.in[1]].dtype != EG_BF16 || g->v[O.in[1]].dtype != EG_BF16 || g->v[f.vexp].dtype != EG_BF16) continue;
        if (g->v[f.vmax].dtype != EG_F32 || g->v[f.vsum].dtype != EG_F32) continue;     // the pass keeps the row statistics in fp32
        if (f.add >= 0 && T1.lbound[lt] > 65536) continue;                              // the pass keeps a table of the mask's key blocks on chip
        if (f.add >= 0 && g->v[f.add].dtype != T1.dtype) continue;                      // one rounding rule for the scores before and after the added operand
        f.qk = t1; f.pv = o; f.q = T1.in[0]; f.k = T1.in[1]; f.v = O.in[1];
        f.lab_s = ls; f.lab_t = lt; f.lab_d = ld; f.lab_dv = ldv;
        taken[t1] = taken[o] = 1;
    }
    return out;
}

// The alternative to the two-stage path for contractions: the join tuples that share an output key run as one
// kernel call whose reduction covers all their blocks, so no partial blocks are written and nothing is left to
// aggregate.  On one GPU that is the same as executing the vertex with its contracted labels unpartitioned.
static bool merges_aggregation(const eg_graph *g, int i)
{
    const Vertex &v = g->v[i];
    if (!g->agg_in_kernel || v.is_input || v.n_in != 2 || v.plan.n_agg <= 1) return false;
    const int kind = eg_route_vertex(g, i);
    return kind == EG_KERNEL_CONTRACT_MFMA || kind == EG_KERNEL_CONTRACT_ALU;
}

// the vertex as the merged kernel call sees it: contracted labels in one piece, one tuple per output block
static Vertex merged_vertex(const Vertex &v)
{
    Vertex m;
    m.dtype = v.dtype; m.bound = v.bound; m.spec = v.spec; m.lx = v.lx; m.ly = v.ly; m.lz = v.lz;
    m.labels = v.labels; m.lbound = v.lbound; m.d = v.d; m.agg = v.agg;
    m.otimes = v.otimes; m.oplus = v.oplus; m.alpha = v.alpha; m.in[0] = v.in[0]; m.in[1] = v.in[1]; m.n_in = v.n_in;
    for (int a : v.agg) m.d[a] = 1;
    m.plan.n_tuples = v.plan.n_tuples / v.plan.n_agg;
    m.plan.n_agg = 1;
    m.plan.n_groups = m.plan.n_tuples;
    m.plan.valid = true;
    return m;
}

// An under-filled contraction with a long reduction (a matrix times a few vectors, a small product of long rows):
// the executor cuts one contracted label further than the vertex's own vector says, as many ways as it takes to
// give the chip's compute units a tile each.  The pieces are ordinary join tuples that write partial slabs, which
// the aggregation adds in ascending order like any others.  Returns the extra factor (a power of two, 1: none).
static int contraction_split(const Vertex &v, const ContractParams &cp, int *label)
{
    const int64_t tiles = ((cp.M + 127) / 128) * ((cp.N + 127) / 128) * cp.n_batch * v.plan.n_tuples;
    if (tiles > 128 || cp.K < 4096) return 1;
    int64_t want = std::min<int64_t>(std::min<int64_t>(512 / tiles, cp.K / 1024), 64);
    int best = -1;
    int64_t be = 0;
    for (int a : v.agg) {
        const int64_t e = v.lbound[a] / v.d[a];
        if (e > be) { be = e; best = a; }
    }
    int c = 1;
    while (best >= 0 && c * 2 <= want && be % (c * 2) == 0 && (be / (c * 2)) % 64 == 0) c *= 2;
    *label = best;
    return c;
}

// the vertex with one contracted label cut c times finer
static Vertex refined_vertex(const Vertex &v, int label, int c)
{
    Vertex m;
    m.dtype = v.dtype; m.bound = v.bound; m.spec = v.spec; m.lx = v.lx; m.ly = v.ly; m.lz = v.lz;
    m.labels = v.labels; m.lbound = v.lbound; m.d = v.d; m.agg = v.agg;
    m.otimes = v.otimes; m.oplus = v.oplus; m.alpha = v.alpha; m.in[0] = v.in[0]; m.in[1] = v.in[1]; m.n_in = v.n_in;
    m.d[label] *= c;
    m.plan.n_tuples = v.plan.n_tuples * c;
    m.plan.n_agg = v.plan.n_agg * c;
    m.plan.n_groups = v.plan.n_groups;
    m.plan.valid = true;
    return m;
}

static Layout make_layout(const eg_graph *g)
{
    const int nv = (int)g->v.size();
    Layout L;
    L.result_off.assign(nv, -1);
    L.partial_off.assign(nv, -1);
    L.split.assign(nv, 1);
    L.split_label.assign(nv, -1);
    L.aux_off.assign(nv, -1);
    // a fused chain runs where its last vertex stands: it reads the chain's outside operands there and writes the
    // result (and the row statistics that are still wanted); the other tensors of the chain never exist
    const std::vector<FuseGroup> groups = find_fusions(g);
    std::vector<int> group_of(nv, -1);
    for (size_t k = 0; k < groups.size(); k++)
        for (int u : groups[k].members()) group_of[u] = (int)k;
    auto reads_of = [&](int i) {                      // what executes at position i reads these tensors
        std::vector<int> in;
        if (group_of[i] >= 0) {
            const FuseGroup &f = groups[group_of[i]];
            if (i == f.anchor()) in = f.reads();
        } else {
            for (int k = 0; k < g->v[i].n_in; k++) in.push_back(g->v[i].in[k]);
        }
        return in;
    };
    std::vector<int> last_use(nv, -1);
    for (int i = 0; i < nv; i++)
        for (int u : reads_of(i)) last_use[u] = i;
    Arena arena;
    for (int i = 0; i < nv; i++) {
        const Vertex &v = g->v[i];
        if (v.is_input) continue;
        if (group_of[i] >= 0) {
            const FuseGroup &f = groups[group_of[i]];
            if (i != f.anchor()) continue;
            for (int u : f.writes())
                if (!g->v[u].is_output) L.result_off[u] = arena.alloc(numel(g->v[u].bound) * dtype_size(g->v[u].dtype));
            if (f.pv >= 0 && f.addend >= 0) {          // the classes of the mask's tiles live for this launch only
                const Vertex &T1 = g->v[f.qk];
                L.aux_off[i] = arena.alloc((int64_t)attention_mask_class_bytes(T1.lbound[f.lab_s], T1.lbound[f.lab_t]));
                arena.release(L.aux_off[i]);
            }
            for (int u : reads_of(i))
                if (last_use[u] == i && L.result_off[u] >= 0) arena.release(L.result_off[u]);
            for (int u : f.writes())
                if (!g->v[u].is_output && last_use[u] < 0) arena.release(L.result_off[u]);
            continue;
        }
        if (!v.is_output) L.result_off[i] = arena.alloc(numel(v.bound) * dtype_size(v.dtype));
        {
            Routed r;
            if (dry_route(g, i, r) == EG_OK) {
                if (r.kind == EG_KERNEL_REDUCE_ROW) L.split[i] = r.rp.split;
                else if ((r.kind == EG_KERNEL_CONTRACT_MFMA || r.kind == EG_KERNEL_CONTRACT_ALU) && !merges_aggregation(g, i))
                    L.split[i] = contraction_split(v, r.cp, &L.split_label[i]);
            }
        }
        const int64_t n_agg = merges_aggregation(g, i) ? 1 : v.plan.n_agg;
        if (n_agg * L.split[i] > 1) {
            L.partial_off[i] = arena.alloc(n_agg * L.split[i] * slab_stride_of(numel(v.bound), n_agg * L.split[i]) * 4);
            arena.release(L.partial_off[i]);          // live only while this vertex runs
        }
        for (int k = 0; k < v.n_in; k++) {
            int u = v.in[k];
            if (last_use[u] == i && L.result_off[u] >= 0 && !(k == 1 && v.in[0] == u)) arena.release(L.result_off[u]);
        }
        if (!v.is_output && last_use[i] < 0) arena.release(L.result_off[i]);   // never consumed
    }
    L.total = arena.top();
    return L;
}

}  // namespace eg

using namespace eg;

// Routing of a vertex with dense row-major operands (what einsum_graph_plan reports and what the workspace
// layout assumes).
int eg::dry_route(const eg_graph *g, int vertex, Routed &r)
{
    const Vertex &v = g->v[vertex];
    static char dummy_buf[64];
    void *aligned = (void *)(((uintptr_t)dummy_buf + 15) & ~(uintptr_t)15);
    Operand X, Y;
    X.ptr = aligned; X.dtype = g->v[v.in[0]].dtype; X.stride = dense_strides(g->v[v.in[0]].bound);
    if (v.n_in > 1) { Y.ptr = aligned; Y.dtype = g->v[v.in[1]].dtype; Y.stride = dense_strides(g->v[v.in[1]].bound); }
    OutSpec out{aligned, 0, (int32_t)v.dtype};
    if (v.plan.n_agg > 1) { out.slab_elems = numel(v.bound); out.dtype = EG_F32; }
    return route(v, X, v.n_in > 1 ? &Y : nullptr, dense_strides(v.bound), out, r);
}

int eg_route_vertex(const eg_graph *g, int vertex)
{
    Routed r;
    if (dry_route(g, vertex, r) != EG_OK) return EG_KERNEL_NONE;
    return r.kind;
}

void eg_release_events(eg_graph *g)
{
    for (void *e : g->ev_start) (void)hipEventDestroy((hipEvent_t)e);
    for (void *e : g->ev_stop) (void)hipEventDestroy((hipEvent_t)e);
    g->ev_start.clear();
    g->ev_stop.clear();
}

static int ensure_events(eg_graph *g, size_t n)
{
    while (g->ev_start.size() < n) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return fail(EG_ERR_HIP, "hipEventCreate failed");
        g->ev_start.push_back((void *)a);
        g->ev_stop.push_back((void *)b);
    }
    return EG_OK;
}

static int launch_routed(Routed &r, void *stream)
{
    switch (r.kind) {
    case EG_KERNEL_CONTRACT_MFMA:
    case EG_KERNEL_CONTRACT_ALU: return launch_contract(r.cp, stream);
    case EG_KERNEL_MAP: return launch_map(r.mp, stream);
    case EG_KERNEL_REDUCE_ROW: return launch_reduce_row(r.rp, stream);
    case EG_KERNEL_GENERIC: return launch_generic(r.gp, stream);
    default: return fail(EG_ERR_BAD_OP, "vertex could not be routed to a kernel");
    }
}

// What the aggregation of tile-ordered partial slabs needs to know about the destination: the contraction's role groups
// once more, with the destination's strides in place of the dense slab's (same labels in the same order, so row, column
// and batch indices mean the same; only which neighbours fuse may differ).
static bool tiles_params(const Vertex &v, const Operand &X, const Operand &Y, const std::vector<int64_t> &zdest, const Routed &r, AggTilesParams &tp)
{
    LabelInfo li = label_info(v, X, &Y, zdest);
    LabelInfo lc = li;
    if (r.swapped)
        for (int l = 0; l < li.nl; l++) { std::swap(lc.inx[l], lc.iny[l]); std::swap(lc.sx[l], lc.sy[l]); }
    ContractParams c2;
    if (!build_contract(v, lc, r.swapped ? Y : X, r.swapped ? X : Y, c2)) return false;
    if (c2.M != r.cp.M || c2.N != r.cp.N || c2.n_batch != r.cp.n_batch) return false;
    memset(&tp, 0, sizeof tp);
    tp.ts = tuple_space(v, li);
    tp.batch = c2.batch; tp.m = c2.m; tp.n = c2.n;
    tp.n_batch = c2.n_batch;
    return true;
}

static int aggregate_into(int oplus, const void *partials, int64_t n_agg, int64_t slab_elems, int64_t slab_stride, void *out, int out_dtype,
                          const std::vector<int64_t> &bound, const std::vector<int64_t> &stride, void *stream)
{
    AggregateParams ap;
    memset(&ap, 0, sizeof ap);
    ap.partials = (const float *)partials;
    ap.n_agg = n_agg;
    ap.slab_elems = slab_elems;
    ap.slab_stride = slab_stride;
    ap.oplus = oplus;
    ap.out_dtype = out_dtype;
    ap.out = out;
    ap.contiguous = stride == dense_strides(bound) ? 1 : 0;
    int nd = 0;
    for (size_t i = 0; i < bound.size(); i++) {
        if (bound[i] == 1) continue;
        if (bound[i] >= (1ll << 31)) return fail(EG_ERR_LIMIT, "aggregate: bound above 2^31");
        ap.dims.ext[nd] = (int32_t)bound[i];
        ap.dims.sz[nd] = stride[i];
        nd++;
    }
    ap.dims.n = nd;
    return launch_aggregate(ap, stream);
}

extern "C" {

int tr_workspace_bytes(eg_graph *g, size_t *bytes)
{
    if (!g || !bytes) return fail(EG_ERR_NULL, "tr_workspace_bytes: NULL argument");
    *bytes = (size_t)make_layout(g).total;
    return EG_OK;
}

int tr_set_fusion(eg_graph *g, int enable)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    g->fuse = enable != 0;
    return EG_OK;
}

int tr_set_fused_aggregation(eg_graph *g, int enable)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    g->agg_in_kernel = enable != 0;
    return EG_OK;
}

int tr_set_tiled_partials(eg_graph *g, int enable)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    g->tiled_partials = enable != 0;
    return EG_OK;
}

int tr_set_fused_attention(eg_graph *g, int enable)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    g->fuse_attention = enable != 0;
    return EG_OK;
}

int tr_set_contract_variant(eg_graph *g, int kernel, int tile_m, int tile_n, int waves)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    if (kernel < 0 || kernel > 2) return fail(EG_ERR_LIMIT, "tr_set_contract_variant: kernel must be 0 (library's choice), 1 (register-staged) or 2 (direct-to-LDS)");
    const bool ok = (tile_m == 0 && tile_n == 0) || (tile_m == 128 && tile_n == 128) || (tile_m == 256 && tile_n == 128) || (tile_m == 256 && tile_n == 256);
    if (!ok) return fail(EG_ERR_LIMIT, "tr_set_contract_variant: tile must be 0 x 0, 128 x 128, 256 x 128 or 256 x 256");
    if (waves != 0 && waves != 4 && waves != 8) return fail(EG_ERR_LIMIT, "tr_set_contract_variant: waves must be 0, 4 or 8");
    g->contract_kernel = kernel;
    g->contract_tile_m = tile_m;
    g->contract_tile_n = tile_n;
    g->contract_waves = waves;
    return EG_OK;
}

int tr_profile_enable(eg_graph *g, int max_launches)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    if (max_launches < 0) return fail(EG_ERR_LIMIT, "max_launches must be >= 0");
    g->profile = max_launches > 0;
    g->launches.clear();
    return g->profile ? ensure_events(g, (size_t)max_launches) : EG_OK;
}

int tr_profile_reset(eg_graph *g)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    g->launches.clear();
    return EG_OK;
}

int tr_profile_count(eg_graph *g)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    return g->profile ? (int)g->launches.size() : 0;
}

int tr_profile_get(eg_graph *g, int i, int *vertex, int *stage, int *kernel, float *ms)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    if (!g->profile || i < 0 || i >= (int)g->launches.size()) return fail(EG_ERR_BAD_VERTEX, "no recorded launch %d", i);
    if (vertex) *vertex = g->launches[i].vertex;
    if (stage) *stage = g->launches[i].stage;
    if (kernel) *kernel = g->launches[i].kernel;
    if (ms) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, (hipEvent_t)g->ev_start[i], (hipEvent_t)g->ev_stop[i]) != hipSuccess)
            return fail(EG_ERR_HIP, "hipEventElapsedTime failed (was the stream synchronised?)");
        *ms = t;
    }
    return EG_OK;
}

}  // extern "C"

// The workspace of tr_execute_static: device memory that belongs to the library, one copy per GPU, held until the
// process ends.  In host code the array's name only stands for the symbol; its device address is looked up once per
// device (scratch_of_current_device) and everything on the host works with that address.
#define EG_STATIC_WORKSPACE_BYTES (32u << 20)
static __device__ __align__(256) unsigned char scratch[EG_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int scratch_of_current_device(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(EG_ERR_HIP, "cannot tell the current device");
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(EG_ERR_HIP, "hipGetSymbolAddress on the static workspace failed: %s", hipGetErrorString(e));
        if ((uintptr_t)p & 255) return fail(EG_ERR_WORKSPACE, "the static workspace is not 256-byte aligned");
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return EG_OK;
}
}  // namespace

// what tr_execute and tr_execute_static share; max_bytes > 0: the workspace is the library's own and holds that much
static int execute_graph(eg_graph *g, eg_relation *const *inputs, int n_inputs, eg_relation *const *outputs, int n_outputs,
                         void *workspace, size_t workspace_bytes, void *hip_stream, size_t max_bytes)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    if (n_inputs != (int)g->inputs.size() || n_outputs != (int)g->outputs.size())
        return fail(EG_ERR_BAD_VERTEX, "graph has %zu inputs and %zu marked outputs; %d and %d relations were given",
                    g->inputs.size(), g->outputs.size(), n_inputs, n_outputs);
    if ((n_inputs && !inputs) || (n_outputs && !outputs)) return fail(EG_ERR_NULL, "relation array is NULL");
    const int nv = (int)g->v.size();
    std::vector<const eg_relation *> bound_rel(nv, nullptr);
    auto check = [&](const eg_relation *r, const Vertex &v, const char *what, int idx) -> int {
        if (!r) return fail(EG_ERR_NULL, "%s relation %d is NULL", what, idx);
        if (r->dtype != v.dtype) return fail(EG_ERR_DTYPE, "%s relation %d: dtype differs from the graph's", what, idx);
        if (r->bound != v.bound) return fail(EG_ERR_BAD_BOUND, "%s relation %d: bound differs from the graph's", what, idx);
        return EG_OK;
    };
    for (int i = 0; i < n_inputs; i++) {
        int rc = check(inputs[i], g->v[g->inputs[i]], "input", i);
        if (rc) return rc;
        bound_rel[g->inputs[i]] = inputs[i];
    }
    for (int i = 0; i < n_outputs; i++) {
        int rc = check(outputs[i], g->v[g->outputs[i]], "output", i);
        if (rc) return rc;
        bound_rel[g->outputs[i]] = outputs[i];
    }
    Layout L = make_layout(g);
    if (max_bytes && (size_t)L.total > max_bytes)
        return fail(EG_ERR_WORKSPACE, "graph needs %lld workspace bytes, the library's static workspace holds %zu: use tr_execute with a workspace of the caller's",
                    (long long)L.total, max_bytes);
    if (L.total > 0) {
        if (!workspace) return fail(EG_ERR_WORKSPACE, "graph needs %lld workspace bytes but workspace is NULL", (long long)L.total);
        if ((uintptr_t)workspace & 255) return fail(EG_ERR_WORKSPACE, "workspace must be 256-byte aligned");
        if ((int64_t)workspace_bytes < L.total)
            return fail(EG_ERR_WORKSPACE, "workspace has %zu bytes, graph needs %lld", workspace_bytes, (long long)L.total);
    }
    char *ws = (char *)workspace;

    // route everything first so that a failure launches nothing
    struct Step { int vertex; Routed r; bool agg; int64_t slabs, stride; const void *partials; void *dst; std::vector<int64_t> dst_stride;
                  bool fused = false; SoftmaxParams sp; bool attn = false; AttnParams ap; bool tiled = false; AggTilesParams tp; };
    std::vector<Step> steps;
    auto operand_of = [&](int u) {
        Operand o;
        const Vertex &pu = g->v[u];
        o.dtype = pu.dtype;
        if (bound_rel[u]) { o.ptr = bound_rel[u]->ptr; o.stride = bound_rel[u]->stride; }
        else { o.ptr = ws + L.result_off[u]; o.stride = dense_strides(pu.bound); }
        return o;
    };
    const std::vector<FuseGroup> groups = find_fusions(g);
    std::vector<int> group_of(nv, -1);
    for (size_t k = 0; k < groups.size(); k++)
        for (int u : groups[k].members()) group_of[u] = (int)k;
    for (int i = 0; i < nv; i++) {
        Vertex &v = g->v[i];
        if (v.is_input) continue;
        if (!v.plan.valid) return fail(EG_ERR_BAD_PARTITION, "vertex %d has no plan", i);
        if (group_of[i] >= 0 && groups[group_of[i]].pv >= 0) {
            const FuseGroup &f = groups[group_of[i]];
            if (i != f.pv) continue;                   // runs as part of the pass that stands at the second contraction
            Step s;
            s.vertex = i;
            s.attn = true;
            s.agg = false;
            AttnParams &ap = s.ap;
            memset(&ap, 0, sizeof ap);
            const Vertex &T1 = g->v[f.qk], &O = g->v[f.pv];
            const int r = (int)T1.lz.size(), nb = r - 2;
            const Operand q = operand_of(f.q), k = operand_of(f.k), vv = operand_of(f.v), o = operand_of(f.pv);
            auto stride_of = [](const std::vector<int> &labels, const Operand &op, int label) -> int64_t {
                for (size_t a = 0; a < labels.size(); a++)
                    if (labels[a] == label) return op.stride[a];
                return 0;
            };
            // the leading (batch) labels of the scores, at most two; O's schema names them O.lx[0..nb)
            int64_t ext[2] = {1, 1}, qs[2] = {0, 0}, ks[2] = {0, 0}, vst[2] = {0, 0}, os[2] = {0, 0};
            for (int a = 0; a < nb; a++) {
                const int at = 2 - nb + a;
                ext[at] = T1.lbound[T1.lz[a]];
                qs[at] = stride_of(T1.lx, q, T1.lz[a]);
                ks[at] = stride_of(T1.ly, k, T1.lz[a]);
                vst[at] = stride_of(O.ly, vv, O.lx[a]);
                os[at] = stride_of(O.lz, o, O.lx[a]);
            }
            if (stride_of(T1.lx, q, f.lab_d) != 1 || stride_of(T1.ly, k, f.lab_d) != 1 || stride_of(O.ly, vv, f.lab_dv) != 1 || stride_of(O.lz, o, f.lab_dv) != 1)
                return fail(EG_ERR_LIMIT, "vertex %d: the one-pass attention needs the head dimension contiguous in Q, K, V and the result; turn tr_set_fused_attention off", i);
            if (T1.lbound[f.lab_s] > INT32_MAX || T1.lbound[f.lab_t] > INT32_MAX || ext[0] > INT32_MAX || ext[1] > INT32_MAX)
                return fail(EG_ERR_LIMIT, "vertex %d: the one-pass attention indexes queries, keys and batch entries with 32 bits", i);
            ap.q = q.ptr; ap.k = k.ptr; ap.v = vv.ptr; ap.o = (void *)o.ptr;
            ap.S = (int32_t)T1.lbound[f.lab_s]; ap.T = (int32_t)T1.lbound[f.lab_t]; ap.D = (int32_t)T1.lbound[f.lab_d];
            ap.nb0 = (int32_t)ext[0]; ap.nb1 = (int32_t)ext[1];
            ap.q_sb0 = qs[0]; ap.q_sb1 = qs[1]; ap.q_ss = stride_of(T1.lx, q, f.lab_s);
            ap.k_sb0 = ks[0]; ap.k_sb1 = ks[1]; ap.k_st = stride_of(T1.ly, k, f.lab_t);
            ap.v_sb0 = vst[0]; ap.v_sb1 = vst[1]; ap.v_st = stride_of(O.ly, vv, O.lx[r - 1]);
            ap.o_sb0 = os[0]; ap.o_sb1 = os[1]; ap.o_ss = stride_of(O.lz, o, O.lx[r - 2]);
            ap.alpha_qk = (float)T1.alpha;
            ap.alpha = 1.f;
            ap.dt_t1 = T1.dtype; ap.dt_t2 = T1.dtype;
            if (f.add >= 0) {
                const Vertex &A = g->v[f.add];
                const Operand m = operand_of(f.addend);
                ap.has_mask = 1; ap.mask = m.ptr; ap.mask_dtype = m.dtype;
                ap.cls = (uint8_t *)(ws + L.aux_off[i]);
                ap.m_ss = stride_of(A.ly, m, r - 2); ap.m_st = stride_of(A.ly, m, r - 1);
                ap.alpha = (float)A.alpha; ap.dt_t2 = A.dtype;
                if (m.dtype != EG_F32 && m.dtype != EG_BF16)
                    return fail(EG_ERR_LIMIT, "vertex %d: the one-pass attention adds an fp32 or bf16 operand; turn tr_set_fused_attention off", i);
            }
            ap.out_dtype = o.dtype;
            steps.push_back(std::move(s));
            continue;
        }
        if (group_of[i] >= 0) {
            const FuseGroup &f = groups[group_of[i]];
            if (i != f.vdiv) continue;                 // runs as part of the pass that stands at the division
            Step s;
            s.vertex = i;
            s.fused = true;
            s.agg = false;
            SoftmaxParams &sp = s.sp;
            memset(&sp, 0, sizeof sp);
            const Vertex &E = g->v[f.vexp], &P = g->v[f.vdiv];
            const int r = (int)E.lx.size();
            const Operand src = operand_of(f.src), res = operand_of(f.vdiv);
            Operand addend, omax, osum;
            LabelInfo li, li2;                          // li: source / added operand / result; li2: row maxima / row sums
            li.nl = li2.nl = r;
            for (int l = 0; l < r; l++) {
                li.ext[l] = li2.ext[l] = P.lbound[l] / P.d[l];
                li.sx[l] = src.stride[l]; li.inx[l] = true;
                li.sz[l] = res.stride[l]; li.inz[l] = true;
            }
            if (f.add >= 0) {
                const Vertex &T = g->v[f.add];
                addend = operand_of(f.addend);
                for (size_t k = 0; k < T.ly.size(); k++) { li.sy[T.ly[k]] = addend.stride[k]; li.iny[T.ly[k]] = true; }
                sp.has_add = 1; sp.add = addend.ptr; sp.dt_add = addend.dtype; sp.dt_t = T.dtype; sp.alpha = (float)T.alpha;
            }
            if (f.emit_max) {
                omax = operand_of(f.vmax);
                for (int l = 0; l + 1 < r; l++) li2.sx[l] = omax.stride[l];
                sp.emit_max = 1; sp.row_max = (void *)omax.ptr; sp.dt_max = omax.dtype;
            }
            if (f.emit_sum) {
                osum = operand_of(f.vsum);
                for (int l = 0; l + 1 < r; l++) li2.sy[l] = osum.stride[l];
                sp.emit_sum = 1; sp.row_sum = (void *)osum.ptr; sp.dt_sum = osum.dtype;
            }
            sp.ts = tuple_space(P, li);                 // the division's partitioning vector is the chain's
            sp.ts2 = tuple_space(P, li2);
            sp.rows_per_block = 1;
            // Row labels that the added operand lacks go last, i.e. vary fastest from one wave to the next: rows that
            // take the same row of the added operand then run next to each other and find it in the cache (otherwise
            // a mask as large as the caches is fetched again for every batch entry and head).
            std::vector<int> order;
            for (int pass = 0; pass < 2; pass++)
                for (int l = 0; l + 1 < r; l++)
                    if ((sp.has_add && li.sy[l] == 0) == (pass == 1)) order.push_back(l);
            for (int l : order) {
                if (li.ext[l] <= 1) continue;
                const int k = sp.rows.n++;
                sp.rows.ext[k] = sp.stats.ext[k] = (int32_t)li.ext[l];
                sp.rows.sx[k] = li.sx[l]; sp.rows.sy[k] = li.sy[l]; sp.rows.sz[k] = li.sz[l];
                sp.stats.sx[k] = li2.sx[l]; sp.stats.sy[k] = li2.sy[l];
                sp.rows_per_block *= li.ext[l];
            }
            sp.stats.n = sp.rows.n;
            sp.n = (int32_t)li.ext[r - 1];
            sp.sx_last = li.sx[r - 1]; sp.sy_last = li.sy[r - 1]; sp.sz_last = li.sz[r - 1];
            sp.dt_src = src.dtype; sp.dt_e = E.dtype; sp.dt_p = res.dtype;
            sp.dt_max = g->v[f.vmax].dtype; sp.dt_sum = g->v[f.vsum].dtype;     // the statistics are rounded as their vertices store them, written or not
            if (!sp.has_add) sp.dt_t = src.dtype;
            sp.src = src.ptr; sp.p = f.emit_div ? (void *)res.ptr : nullptr;
            sp.emit_p = f.emit_div ? 1 : 0;
            sp.n_tuples = P.plan.n_tuples;
            if (!f.tails.empty()) {
                // strides, label by label, of the tensors the tails read (entries 0, 1) and write (2 + k); row tensors lack the last label
                std::vector<std::vector<int64_t>> st(kSoftmaxMore, std::vector<int64_t>(r, 0));
                sp.n_ext = (int32_t)f.ext.size();
                sp.n_tail = (int32_t)f.tails.size();
                for (size_t e = 0; e < f.ext.size(); e++) {
                    const Operand o = operand_of(f.ext[e]);
                    sp.ext[e] = o.ptr; sp.dt_ext[e] = o.dtype;
                    for (int l = 0; l < r; l++) st[e][l] = o.stride[l];
                }
                for (size_t k = 0; k < f.tails.size(); k++) {
                    const Vertex &T = g->v[f.tails[k]];
                    SoftmaxTail &tl = sp.tail[k];
                    tl.op = T.otimes; tl.alpha = (float)T.alpha;
                    tl.a = f.tail_a[k]; tl.b = T.n_in == 2 ? f.tail_b[k] : -1;
                    tl.row = f.tail_row[k]; tl.dt = T.dtype; tl.emit = f.tail_emit[k];
                    if (tl.emit) {
                        const Operand o = operand_of(f.tails[k]);
                        tl.out = (void *)o.ptr;
                        for (size_t l = 0; l < o.stride.size() && l < (size_t)r; l++) st[kSoftmaxExt + k][l] = o.stride[l];
                    }
                }
                for (int e = 0; e < kSoftmaxMore; e++) {
                    sp.more_last[e] = (e >= kSoftmaxExt && e - kSoftmaxExt < sp.n_tail && sp.tail[e - kSoftmaxExt].row) ? 0 : st[e][r - 1];
                    int k = 0, n = 0;
                    for (int l : order)
                        if (li.ext[l] > 1) sp.more_rows[e][k++] = st[e][l];
                    for (int l = 0; l < r; l++)
                        if (P.d[l] > 1) sp.more_step[e][n++] = li.ext[l] * st[e][l];
                }
            }
            steps.push_back(std::move(s));
            continue;
        }
        Step s;
        s.vertex = i;
        const bool merged = merges_aggregation(g, i);
        const bool refined = !merged && L.split_label[i] >= 0 && L.split[i] > 1;
        const Vertex vm = merged ? merged_vertex(v) : refined ? refined_vertex(v, L.split_label[i], L.split[i]) : Vertex();
        const Vertex &vr = merged || refined ? vm : v;   // what is routed: the vertex, its merged form, or its finer cut
        Operand X = operand_of(v.in[0]), Y;
        if (v.n_in > 1) Y = operand_of(v.in[1]);
        Operand Z = operand_of(i);
        s.dst = (void *)Z.ptr;
        s.dst_stride = Z.stride;
        s.slabs = refined ? vr.plan.n_agg : vr.plan.n_agg * L.split[i];
        s.agg = s.slabs > 1;
        OutSpec out;
        std::vector<int64_t> zstride;
        if (s.agg) {
            s.partials = ws + L.partial_off[i];
            out.ptr = (void *)s.partials;
            out.slab_elems = slab_stride_of(numel(v.bound), s.slabs);
            out.dtype = EG_F32;
            zstride = dense_strides(v.bound);
        } else {
            s.partials = nullptr;
            out.ptr = s.dst;
            out.slab_elems = 0;
            out.dtype = v.dtype;
            zstride = Z.stride;
        }
        int rc = route(vr, X, v.n_in > 1 ? &Y : nullptr, zstride, out, s.r, refined ? 1 : L.split[i]);
        if (rc) return rc;
        const Vertex *routed = &vr;
        if (merged && s.r.kind != EG_KERNEL_CONTRACT_MFMA && s.r.kind != EG_KERNEL_CONTRACT_ALU)
            return fail(EG_ERR_LIMIT, "vertex %d: the bound relations' strides leave no contraction kernel for the merged aggregation; turn tr_set_fused_aggregation off", i);
        if (L.split[i] > 1 && s.r.kind != EG_KERNEL_REDUCE_ROW &&
            !(refined && (s.r.kind == EG_KERNEL_CONTRACT_MFMA || s.r.kind == EG_KERNEL_CONTRACT_ALU))) {
            // the bound relations' strides sent this vertex to another kernel than the layout assumed:
            // run it unsplit, writing the tensor directly when nothing else needs aggregating
            s.slabs = v.plan.n_agg;
            s.agg = s.slabs > 1;
            if (!s.agg) { out.ptr = s.dst; out.slab_elems = 0; out.dtype = v.dtype; zstride = Z.stride; }
            rc = route(v, X, v.n_in > 1 ? &Y : nullptr, zstride, out, s.r, 1);
            if (rc) return rc;
            routed = &v;
        }
        if (s.r.kind == EG_KERNEL_REDUCE_ROW && !refined && s.r.rp.split != L.split[i]) s.r.rp.split = L.split[i];
        s.stride = out.slab_elems;                 // what the join kernel was given
        if (s.r.kind == EG_KERNEL_CONTRACT_MFMA || s.r.kind == EG_KERNEL_CONTRACT_ALU) {
            s.r.cp.force_kernel = g->contract_kernel;
            s.r.cp.force_tile_m = g->contract_tile_m;
            s.r.cp.force_tile_n = g->contract_tile_n;
            s.r.cp.force_waves = g->contract_waves;
        }
        // Partial slabs of the direct-to-LDS contraction kernel in tile order when its tiles are whole: the slab has the same
        // size, only the order of its elements is a matter between that kernel and the aggregation that follows it.  The join
        // kernel saves some 5 us per tile (no staging through LDS), the aggregation of tile-ordered slabs runs at 0.70 of the
        // memory rate where the dense one reaches up to 0.84: taken where a tile's reduction is short enough for the 5 us to
        // count (up to 4096; config 6's product with 12800 per tile lost 0.5 % per step with it).
        if (s.agg && g->tiled_partials && s.r.kind == EG_KERNEL_CONTRACT_MFMA && s.r.cp.K <= 4096 && contract_takes_dma(s.r.cp)) {
            const Vertex &vu = *routed;
            int tm = 0, tn = 0, nw = 0;
            contract_dma_variant(s.r.cp, tm, tn, nw);
            const ContractParams &cp = s.r.cp;
            if (tm > 0 && cp.M % tm == 0 && cp.N % tn == 0 && vu.plan.n_tuples % s.slabs == 0 && v.n_in == 2 &&
                tiles_params(vu, X, Y, Z.stride, s.r, s.tp)) {
                AggTilesParams &tp = s.tp;
                tp.tm = tm; tp.tn = tn; tp.nw = nw;
                tp.tiles_m = (int32_t)(cp.M / tm); tp.tiles_n = (int32_t)(cp.N / tn);
                tp.tiles = vu.plan.n_tuples / s.slabs * cp.n_batch * tp.tiles_m * tp.tiles_n;
                tp.partials = (const float *)s.partials; tp.n_agg = s.slabs; tp.slab_stride = s.stride;
                tp.out = s.dst; tp.out_dtype = v.dtype;
                if (tp.tiles * tm * tn == numel(v.bound)) {
                    s.tiled = true;
                    s.r.cp.tile_order = 1;
                }
            }
        }
        steps.push_back(std::move(s));
    }
    hipStream_t st = (hipStream_t)hip_stream;
    auto timed = [&](int vertex, int stage, int kernel, int64_t slabs, auto &&fn) -> int {
        const size_t idx = g->launches.size();
        const bool rec = g->profile && idx < g->ev_start.size();
        if (rec && hipEventRecord((hipEvent_t)g->ev_start[idx], st) != hipSuccess) return fail(EG_ERR_HIP, "hipEventRecord failed");
        int rc = fn();
        if (rc) return rc;
        if (rec) {
            if (hipEventRecord((hipEvent_t)g->ev_stop[idx], st) != hipSuccess) return fail(EG_ERR_HIP, "hipEventRecord failed");
            g->launches.push_back({vertex, stage, kernel, slabs});
        }
        return EG_OK;
    };
    // every launcher once without launching: limits that only show when the grid is sized (tile counts, row lengths,
    // 32-bit grid bounds, kernel attributes) are found before anything has been enqueued
    {
        struct Guard { Guard() { set_validate_only(true); } ~Guard() { set_validate_only(false); } } guard;
        for (Step &s : steps) {
            const Vertex &v = g->v[s.vertex];
            int rc = s.attn ? launch_attention(s.ap, hip_stream) : s.fused ? launch_softmax_rows(s.sp, hip_stream) : launch_routed(s.r, hip_stream);
            if (rc) return rc;
            if (s.agg) {
                rc = s.tiled ? launch_aggregate_tiles(s.tp, hip_stream)
                             : aggregate_into(v.oplus, s.partials, s.slabs, numel(v.bound), s.stride, s.dst, v.dtype, v.bound, s.dst_stride, hip_stream);
                if (rc) return rc;
            }
        }
    }
    for (Step &s : steps) {
        const Vertex &v = g->v[s.vertex];
        int rc = s.attn  ? timed(s.vertex, 0, EG_KERNEL_ATTENTION_FUSED, 0, [&] { return launch_attention(s.ap, hip_stream); })
               : s.fused ? timed(s.vertex, 0, EG_KERNEL_SOFTMAX_FUSED, 0, [&] { return launch_softmax_rows(s.sp, hip_stream); })
                         : timed(s.vertex, 0, s.r.kind, s.agg ? s.slabs : 0, [&] { return launch_routed(s.r, hip_stream); });
        if (rc) return rc;
        if (s.agg) {
            rc = timed(s.vertex, 1, s.tiled ? EG_KERNEL_AGGREGATE_TILES : EG_KERNEL_NONE, s.slabs, [&] {
                return s.tiled ? launch_aggregate_tiles(s.tp, hip_stream)
                               : aggregate_into(v.oplus, s.partials, s.slabs, numel(v.bound), s.stride, s.dst, v.dtype, v.bound, s.dst_stride, hip_stream);
            });
            if (rc) return rc;
        }
    }
    return EG_OK;
}

extern "C" {

int tr_profile_get_slabs(eg_graph *g, int i, int64_t *slabs)
{
    if (!g || !slabs) return fail(EG_ERR_NULL, "tr_profile_get_slabs: NULL argument");
    if (!g->profile || i < 0 || i >= (int)g->launches.size()) return fail(EG_ERR_BAD_VERTEX, "no recorded launch %d", i);
    *slabs = g->launches[i].slabs;
    return EG_OK;
}

int tr_execute(eg_graph *g, eg_relation *const *inputs, int n_inputs, eg_relation *const *outputs, int n_outputs,
               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return execute_graph(g, inputs, n_inputs, outputs, n_outputs, workspace, workspace_bytes, hip_stream, 0);
}

int tr_execute_static(eg_graph *g, eg_relation *const *inputs, int n_inputs, eg_relation *const *outputs, int n_outputs, void *hip_stream)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    void *ws = nullptr;
    int rc = scratch_of_current_device(&ws);
    if (rc) return rc;
    return execute_graph(g, inputs, n_inputs, outputs, n_outputs, ws, EG_STATIC_WORKSPACE_BYTES, hip_stream, EG_STATIC_WORKSPACE_BYTES);
}

size_t tr_static_workspace_bytes(void) { return EG_STATIC_WORKSPACE_BYTES; }

int tr_aggregate(eg_agg oplus, const void *partials, int64_t n_agg, int64_t slab_elems, eg_relation *out, void *hip_stream)
{
    if (!partials || !out) return fail(EG_ERR_NULL, "tr_aggregate: NULL argument");
    if (oplus != EG_AGG_SUM && oplus != EG_AGG_MAX) return fail(EG_ERR_BAD_OP, "tr_aggregate: (+) must be SUM or MAX");
    if (n_agg < 1) return fail(EG_ERR_BAD_PARTITION, "tr_aggregate: n_agg must be >= 1");
    if (slab_elems != numel(out->bound)) return fail(EG_ERR_BAD_BOUND, "tr_aggregate: slab_elems %lld differs from the output's %lld elements",
                                                      (long long)slab_elems, (long long)numel(out->bound));
    if ((uintptr_t)partials & 15) return fail(EG_ERR_WORKSPACE, "tr_aggregate: partials must be 16-byte aligned");
    return aggregate_into((int)oplus, partials, n_agg, slab_elems, slab_elems, out->ptr, out->dtype, out->bound, out->stride, hip_stream);
}

}  // extern "C"
