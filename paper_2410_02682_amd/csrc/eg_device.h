// Device helpers shared by the kernels: dtype conversion, the scalar functions (x), tuple decoding.
#pragma once

#include <hip/hip_runtime.h>

#include "eg_internal.h"

namespace eg {

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest, ties to even (the hardware conversion of gfx950).
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    __bf16 h = (__bf16)f;
    return *(uint16_t *)&h;
}

typedef __bf16 eg_bf16x2 __attribute__((ext_vector_type(2)));
typedef float eg_f32x2 __attribute__((ext_vector_type(2)));

// two fp32 -> one dword holding two bf16 (a in the low half)
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    eg_f32x2 v = {a, b};
    eg_bf16x2 r = __builtin_convertvector(v, eg_bf16x2);
    return *(uint32_t *)&r;
}

__device__ __forceinline__ float load_elem(const void *p, int dt, int64_t off)
{
    return dt == EG_BF16 ? bf16_to_f32(((const uint16_t *)p)[off]) : ((const float *)p)[off];
}

__device__ __forceinline__ void store_elem(void *p, int dt, int64_t off, float v)
{
    if (dt == EG_BF16) ((uint16_t *)p)[off] = f32_to_bf16(v);
    else ((float *)p)[off] = v;
}

// Loads 8 consecutive elements as fp32 (16-byte aligned start).
__device__ __forceinline__ void load8(const void *p, int dt, int64_t off, float (&v)[8])
{
    if (dt == EG_BF16) {
        uint4 r = *(const uint4 *)((const uint16_t *)p + off);
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
        v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
        v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
    } else {
        float4 a = *(const float4 *)((const float *)p + off);
        float4 b = *(const float4 *)((const float *)p + off + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

__device__ __forceinline__ void store8(void *p, int dt, int64_t off, const float (&v)[8])
{
    if (dt == EG_BF16) {
        uint4 r;
        r.x = pack_bf16x2(v[0], v[1]);
        r.y = pack_bf16x2(v[2], v[3]);
        r.z = pack_bf16x2(v[4], v[5]);
        r.w = pack_bf16x2(v[6], v[7]);
        *(uint4 *)((uint16_t *)p + off) = r;
    } else {
        *(float4 *)((float *)p + off) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4 *)((float *)p + off + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
}

// exp(x - y) where the result is stored as bf16: one multiply-add into the hardware's base-2 exponential.
// y * log2(e) is rounded once, which puts an absolute error of about |y| * 2^-24 into the exponent, far below
// the 2^-9 half-ulp of the stored value.  The fused softmax pass uses the same expression, so it agrees bit
// for bit with the separate vertex.
constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float exp_sub_scaled(float x, float neg_y_log2e) { return __builtin_amdgcn_exp2f(fmaf(x, kLog2e, neg_y_log2e)); }
__device__ __forceinline__ float exp_sub_fast(float x, float y) { return exp_sub_scaled(x, -(y * kLog2e)); }

// Rounds two fp32 values to bf16 and back with one conversion instruction.
__device__ __forceinline__ void round_pair_bf16(float &a, float &b)
{
    const uint32_t pk = pack_bf16x2(a, b);
    a = __uint_as_float(pk << 16);
    b = __uint_as_float(pk & 0xffff0000u);
}

// The scalar function (x) of a vertex (Section 3 of the paper: any scalar function of the joined values).
// OP >= 0 fixes the function at compile time; OP = -1 reads it from `op`.  FAST selects the hardware
// exponential (relative error about |x| * 6e-8) and reciprocal (1 ulp), used only where the result is
// stored as bf16.
template <int OP, bool FAST>
__device__ __forceinline__ float otimes_t(int op, float x, float y, float alpha)
{
    const int o = OP >= 0 ? OP : op;
    switch (o) {
    case EG_MUL: return alpha * (x * y);
    case EG_ADD: return alpha * x + y;
    case EG_SUB: return alpha * (x - y);
    case EG_DIV: return FAST ? x * __frcp_rn(y) : x / y;
    case EG_SQDIFF: return (x - y) * (x - y);
    case EG_ABSDIFF: return fabsf(x - y);
    case EG_EXP_SUB: return FAST ? exp_sub_fast(x, y) : expf(x - y);
    case EG_RELU_GRAD: return y > 0.f ? x : 0.f;
    case EG_SILU_MUL: return (x / (1.f + (FAST ? __expf(-x) : expf(-x)))) * y;
    case EG_IDENT: return x;
    case EG_SCALE: return alpha * x;
    case EG_RELU: return x > 0.f ? x : 0.f;
    case EG_EXP: return FAST ? __expf(x) : expf(x);
    case EG_LOG: return logf(x);
    default: return 0.f;
    }
}

__device__ __forceinline__ float otimes_eval(int op, float x, float y, float alpha) { return otimes_t<-1, false>(op, x, y, alpha); }

template <int OPLUS>
__device__ __forceinline__ float oplus_t(int oplus, float a, float b)
{
    const int o = OPLUS >= 0 ? OPLUS : oplus;
    return o == EG_AGG_MAX ? fmaxf(a, b) : a + b;
}

__device__ __forceinline__ float oplus_identity(int oplus) { return oplus == EG_AGG_MAX ? -INFINITY : 0.f; }
__device__ __forceinline__ float oplus_eval(int oplus, float a, float b) { return oplus == EG_AGG_MAX ? fmaxf(a, b) : a + b; }

// Tuple t -> base offsets of its X / Y / Z blocks and its aggIdx (row-major over I(d), last label fastest).
__device__ __forceinline__ void decode_tuple(const TupleSpace &ts, int64_t t, int64_t &ox, int64_t &oy, int64_t &oz, int64_t &agg)
{
    ox = oy = oz = agg = 0;
    uint32_t rem = (uint32_t)t;
    for (int l = ts.n - 1; l >= 0; l--) {
        uint32_t dd = (uint32_t)ts.d[l];
        uint32_t q = rem / dd, k = rem - q * dd;
        rem = q;
        ox += (int64_t)k * ts.step_x[l];
        oy += (int64_t)k * ts.step_y[l];
        oz += (int64_t)k * ts.step_z[l];
        agg += (int64_t)k * ts.agg_w[l];
    }
}

// Tuple t -> index of its output block (row-major over the partitioned labels that are not aggregated).
__device__ __forceinline__ int64_t tuple_group(const TupleSpace &ts, int64_t t)
{
    int64_t g = 0;
    uint32_t rem = (uint32_t)t;
    for (int l = ts.n - 1; l >= 0; l--) {
        uint32_t dd = (uint32_t)ts.d[l];
        uint32_t q = rem / dd, k = rem - q * dd;
        rem = q;
        g += (int64_t)k * ts.grp_w[l];
    }
    return g;
}

// ... and back: output block index -> Z offset of the block.
__device__ __forceinline__ int64_t group_offset_z(const TupleSpace &ts, int64_t g)
{
    int64_t oz = 0;
    uint32_t rem = (uint32_t)g;
    for (int l = ts.n - 1; l >= 0; l--) {
        if (ts.grp_w[l] == 0) continue;                // an aggregated label: no part of the block index
        uint32_t dd = (uint32_t)ts.d[l];
        uint32_t q = rem / dd, k = rem - q * dd;
        rem = q;
        oz += (int64_t)k * ts.step_z[l];
    }
    return oz;
}

// Flat index within a collapsed index space -> offsets in X / Y / Z.
__device__ __forceinline__ void decode_dims(const StridedDims &d, int64_t e, int64_t &ox, int64_t &oy, int64_t &oz)
{
    for (int i = d.n - 1; i >= 0; i--) {
        int64_t q = e / d.ext[i], k = e - q * d.ext[i];
        e = q;
        ox += k * d.sx[i];
        oy += k * d.sy[i];
        oz += k * d.sz[i];
    }
}

}  // namespace eg
