// Measured ceilings of the box, reported next to the datasheet peaks: a register-resident bf16 MFMA loop
// (no memory traffic at all), a plain streaming copy, 16 bytes per lane, and a read-mostly stream (N pieces in, one out).
// None is part of the einsum path.
#include <hip/hip_runtime.h>

#include "eg_internal.h"

namespace eg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void k_mfma_ceiling(float *sink, int iters)
{
    bf16x8 a, b;
    for (int i = 0; i < 8; i++) { a[i] = (__bf16)(float)(threadIdx.x & 3); b[i] = (__bf16)(float)(i & 1); }
    f32x16 acc[8];
    for (int t = 0; t < 8; t++)
        for (int r = 0; r < 16; r++) acc[t][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int t = 0; t < 8; t++) acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t], 0, 0, 0);
    }
    float s = 0.f;
    for (int t = 0; t < 8; t++)
        for (int r = 0; r < 16; r++) s += acc[t][r];
    if (s == -1.f) sink[0] = s;      // never true: keeps the loop alive
}

// The same loop on operands that look like data: four A and four B fragments of pseudo-random bf16 values per lane
// (sign and mantissa bits from a hash, magnitudes around one), 16 accumulator tiles.  What the matrix pipes deliver
// depends on how many operand bits toggle, because the chip lowers its clock under the power they draw; this is the
// rate to hold a contraction on real operands against.
__global__ __launch_bounds__(256) void k_mfma_ceiling_random(float *sink, int iters, unsigned seed)
{
    bf16x8 a[4], b[4];
    unsigned h = (threadIdx.x + 1) * 2654435761u ^ seed ^ (blockIdx.x * 40503u);
    for (int s = 0; s < 4; s++)
        for (int i = 0; i < 8; i++) {
            h = h * 1664525u + 1013904223u;
            const unsigned short ua = (unsigned short)(0x3c00 + ((h >> 16) & 0x83ff));
            h = h * 1664525u + 1013904223u;
            const unsigned short ub = (unsigned short)(0x3c00 + ((h >> 16) & 0x83ff));
            a[s][i] = __builtin_bit_cast(__bf16, ua);
            b[s][i] = __builtin_bit_cast(__bf16, ub);
        }
    f32x16 acc[4][4];
    for (int i = 0; i < 4; i++)
        for (int j = 0; j < 4; j++)
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; i++)
        for (int j = 0; j < 4; j++)
            for (int r = 0; r < 16; r++) s += acc[i][j][r];
    if (s == -1.2345f) sink[0] = s;  // never true: keeps the loop alive
}

// Register-resident chains of the instruction pair the distance kernels live on: subtract, then fused
// multiply-add of the difference with itself into an accumulator (16 independent accumulators per lane).
__global__ __launch_bounds__(256) void k_valu_ceiling(float *sink, int iters, float x)
{
    float a[16];
    for (int i = 0; i < 16; i++) a[i] = threadIdx.x * 0.001f + i;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int r = 0; r < 4; r++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const float d = a[i] - x;
                a[i] = __builtin_fmaf(d, d, a[i]);
            }
    }
    float s = 0.f;
    for (int i = 0; i < 16; i++) s += a[i];
    if (s == 12345.678f) sink[0] = s;  // never true for the x the launcher passes: keeps the loop alive
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One 16-byte vector per lane, streaming (non-temporal) load and store: the fastest plain copy found on this part.
__global__ __launch_bounds__(256) void k_copy_ceiling(u32x4 *dst, const u32x4 *src, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}


// N streams read, one written, 16 bytes per lane and stream: the traffic shape of an aggregation of N partial slabs, without
// its arithmetic (the vectors are combined with exclusive-or).  What memory gives to a read-mostly kernel.
template <int N>
__global__ __launch_bounds__(256) void k_read_ceiling(u32x4 *dst, const u32x4 *src, int64_t n16)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    u32x4 v[N];
#pragma unroll
    for (int k = 0; k < N; k++) v[k] = __builtin_nontemporal_load(src + k * n16 + i);
    u32x4 r = v[0];
#pragma unroll
    for (int k = 1; k < N; k++) r ^= v[k];
    __builtin_nontemporal_store(r, dst + i);
}

}  // namespace eg

extern "C" {

// Launches `waves_per_simd` waves on every SIMD of `cus` compute units, each issuing iters*8 independent
// 32x32x16 bf16 MFMAs from registers.  *flops receives the floating-point operation count of the launch.
// sink: device, at least 4 bytes (never written).
int eg_ceiling_mfma_bf16(void *sink, int cus, int waves_per_simd, int iters, double *flops, void *hip_stream)
{
    if (!sink || !flops) return eg::fail(EG_ERR_NULL, "eg_ceiling_mfma_bf16: NULL argument");
    if (cus < 1 || waves_per_simd < 1 || waves_per_simd > 2 || iters < 1) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_mfma_bf16: bad launch shape");
    const int wgs = cus * waves_per_simd;
    hipLaunchKernelGGL(eg::k_mfma_ceiling, dim3(wgs), dim3(256), 0, (hipStream_t)hip_stream, (float *)sink, iters);
    if (hipGetLastError() != hipSuccess) return eg::fail(EG_ERR_HIP, "k_mfma_ceiling launch failed");
    *flops = (double)wgs * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 16);
    return EG_OK;
}

// As eg_ceiling_mfma_bf16, on pseudo-random operands (16 MFMAs per wave and iteration); one wave per SIMD only,
// the loop holds 256 accumulator registers.
int eg_ceiling_mfma_bf16_random(void *sink, int cus, int iters, double *flops, void *hip_stream)
{
    if (!sink || !flops) return eg::fail(EG_ERR_NULL, "eg_ceiling_mfma_bf16_random: NULL argument");
    if (cus < 1 || iters < 1) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_mfma_bf16_random: bad launch shape");
    hipLaunchKernelGGL(eg::k_mfma_ceiling_random, dim3(cus), dim3(256), 0, (hipStream_t)hip_stream, (float *)sink, iters, 7u);
    if (hipGetLastError() != hipSuccess) return eg::fail(EG_ERR_HIP, "k_mfma_ceiling_random launch failed");
    *flops = (double)cus * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
    return EG_OK;
}

// Launches `waves_per_simd` (1, 2 or 4) waves on every SIMD of `cus` compute units, each lane running iters*64
// subtract + fused-multiply-add pairs from registers.  *pairs receives the number of pairs of the launch.
int eg_ceiling_valu_f32(void *sink, int cus, int waves_per_simd, int iters, double *pairs, void *hip_stream)
{
    if (!sink || !pairs) return eg::fail(EG_ERR_NULL, "eg_ceiling_valu_f32: NULL argument");
    if (cus < 1 || (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4) || iters < 1) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_valu_f32: bad launch shape");
    const int wgs = cus * waves_per_simd;
    hipLaunchKernelGGL(eg::k_valu_ceiling, dim3(wgs), dim3(256), 0, (hipStream_t)hip_stream, (float *)sink, iters, 1.0001f);
    if (hipGetLastError() != hipSuccess) return eg::fail(EG_ERR_HIP, "k_valu_ceiling launch failed");
    *pairs = (double)wgs * 256.0 * iters * 64.0;
    return EG_OK;
}

// Copies `bytes` (a multiple of 16, both pointers 16-byte aligned, device) with a grid-stride loop.
int eg_ceiling_copy(void *dst, const void *src, int64_t bytes, void *hip_stream)
{
    if (!dst || !src) return eg::fail(EG_ERR_NULL, "eg_ceiling_copy: NULL argument");
    if (bytes < 16 || bytes % 16 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_copy: size/alignment");
    const int64_t n16 = bytes / 16, wgs = (n16 + 255) / 256;
    if (wgs >= (1ll << 31)) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_copy: too large for one launch");
    hipLaunchKernelGGL(eg::k_copy_ceiling, dim3((unsigned)wgs), dim3(256), 0, (hipStream_t)hip_stream, (eg::u32x4 *)dst, (const eg::u32x4 *)src, n16);
    if (hipGetLastError() != hipSuccess) return eg::fail(EG_ERR_HIP, "k_copy_ceiling launch failed");
    return EG_OK;
}


// Reads `streams` (2, 8 or 16) consecutive pieces of `bytes` each from src and writes one piece of `bytes` to dst
// (bytes: a multiple of 16; pointers device, 16-byte aligned; src holds streams * bytes).
int eg_ceiling_read(void *dst, const void *src, int streams, int64_t bytes, void *hip_stream)
{
    if (!dst || !src) return eg::fail(EG_ERR_NULL, "eg_ceiling_read: NULL argument");
    if (bytes < 16 || bytes % 16 || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_read: size/alignment");
    const int64_t n16 = bytes / 16, wgs = (n16 + 255) / 256;
    if (wgs >= (1ll << 31)) return eg::fail(EG_ERR_LIMIT, "eg_ceiling_read: too large for one launch");
    hipStream_t st = (hipStream_t)hip_stream;
    if (streams == 2) hipLaunchKernelGGL(eg::k_read_ceiling<2>, dim3((unsigned)wgs), dim3(256), 0, st, (eg::u32x4 *)dst, (const eg::u32x4 *)src, n16);
    else if (streams == 8) hipLaunchKernelGGL(eg::k_read_ceiling<8>, dim3((unsigned)wgs), dim3(256), 0, st, (eg::u32x4 *)dst, (const eg::u32x4 *)src, n16);
    else if (streams == 16) hipLaunchKernelGGL(eg::k_read_ceiling<16>, dim3((unsigned)wgs), dim3(256), 0, st, (eg::u32x4 *)dst, (const eg::u32x4 *)src, n16);
    else return eg::fail(EG_ERR_LIMIT, "eg_ceiling_read: 2, 8 or 16 streams");
    if (hipGetLastError() != hipSuccess) return eg::fail(EG_ERR_HIP, "k_read_ceiling launch failed");
    return EG_OK;
}

}  // extern "C"
