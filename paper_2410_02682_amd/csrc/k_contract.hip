// Block contraction on MFMA: the per-block kernel K of Section 4.3 of the paper for (x) = multiply,
// (+) = sum, i.e. Z'[l_Z] = sum over l_agg of X^{kX}[l_X] * Y^{kY}[l_Y] on one joined pair of blocks.
//
// Every tuple of the join is viewed as a strided batched matrix product: labels in X, Y and Z are batch
// labels, labels in X and Z form M, labels in Y and Z form N, labels in X and Y only form K.  One launch
// covers all tuples: workgroup -> (tuple, batch index, M tile, N tile).  Tiles are staged through LDS in
// 16-byte chunks with an XOR swizzle; an operand that is contiguous along M or N instead of K is
// transposed in registers on its way into LDS, so the MFMA feed is identical for every layout.
// fp32 accumulation; the epilogue either writes fp32 partial blocks (slab aggIdx) or casts once to the
// vertex dtype.
#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>

#include "eg_device.h"

namespace eg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int BM_, int BN_, int WM_, int WN_, bool BF16_>
struct Cfg {
    static constexpr int BM = BM_, BN = BN_, WM = WM_, WN = WN_;
    static constexpr bool BF16 = BF16_;
    static constexpr int ESZ = BF16_ ? 2 : 4;             // element bytes
    static constexpr int EPC = 16 / ESZ;                  // elements per 16-byte chunk
    static constexpr int BK = 8 * EPC;                    // 8 chunks = 128 bytes per tile row
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int THREADS = WAVES_M * WAVES_N * 64;
    static constexpr int MT = WM / 32, NT = WN / 32;      // 32x32 MFMA tiles per wave
    static constexpr int NVA = BM * 8 / THREADS;          // 16-byte vectors per thread per stage
    static constexpr int NVB = BN * 8 / THREADS;
    static constexpr int LDS_A = BM * 128, LDS_B = BN * 128;
    static constexpr int LDS_BYTES = 2 * (LDS_A + LDS_B);
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0, "tile shape");
    static_assert((BM * 8) % THREADS == 0 && (BN * 8) % THREADS == 0, "tile / thread split");
    static_assert(THREADS % 8 == 0 && THREADS % (BM / EPC) == 0 && THREADS % (BN / EPC) == 0, "loader split");
};

// Swizzled byte offset of 16-byte chunk `chunk` (0..7) in tile row `row`.
__device__ __forceinline__ int lds_off(int row, int chunk) { return row * 128 + ((chunk ^ ((row ^ (row >> 3)) & 7)) << 4); }

// index within a role group -> element offsets in the two tensors that carry the group
__device__ __forceinline__ void decode_group(const DimList &g, int64_t idx, int64_t &o0, int64_t &o1)
{
    o0 = o1 = 0;
    if (g.n == 1) {
        o0 = idx * g.s0[0];
        o1 = idx * g.s1[0];
        return;
    }
    uint32_t rem = (uint32_t)idx;
    for (int i = g.n - 1; i >= 0; i--) {
        uint32_t e = (uint32_t)g.ext[i], q = rem / e, k = rem - q * e;
        rem = q;
        o0 += (int64_t)k * g.s0[i];
        o1 += (int64_t)k * g.s1[i];
    }
}

// Gathers element j of each of the NV register vectors (one k-row each) into consecutive k order.
template <int NV, bool BF16>
__device__ __forceinline__ void transpose_store(const uint4 (&v)[NV], char *lds_tile, int row0, int kfirst)
{
    constexpr int EPC = BF16 ? 8 : 4;
    constexpr int G = NV < EPC ? NV : EPC;          // k-values per LDS write (stay inside one 16-byte chunk)
#pragma unroll
    for (int j = 0; j < EPC; j++) {
        const int row = row0 + j;
#pragma unroll
        for (int g0 = 0; g0 < NV; g0 += G) {
            const int k = kfirst + g0;              // first k of this group within the stage
            char *dst = lds_tile + lds_off(row, k / EPC) + (k % EPC) * (BF16 ? 2 : 4);
            if (BF16) {
                uint32_t w[G / 2];
#pragma unroll
                for (int q = 0; q < G / 2; q++) {
                    const uint32_t *a = (const uint32_t *)&v[g0 + 2 * q];
                    const uint32_t *b = (const uint32_t *)&v[g0 + 2 * q + 1];
                    uint32_t lo = (j & 1) ? (a[j >> 1] >> 16) : (a[j >> 1] & 0xffffu);
                    uint32_t hi = (j & 1) ? (b[j >> 1] & 0xffff0000u) : (b[j >> 1] << 16);
                    w[q] = lo | hi;
                }
                if (G == 8) *(uint4 *)dst = make_uint4(w[0], w[1], w[2], w[3]);
                else if (G == 4) *(uint2 *)dst = make_uint2(w[0], w[1]);
                else *(uint32_t *)dst = w[0];
            } else {
                uint32_t w[G];
#pragma unroll
                for (int q = 0; q < G; q++) w[q] = ((const uint32_t *)&v[g0 + q])[j];
                if (G == 4) *(uint4 *)dst = make_uint4(w[0], w[1], w[2], w[3]);
                else if (G == 2) *(uint2 *)dst = make_uint2(w[0], w[1]);
                else *(uint32_t *)dst = w[0];
            }
        }
    }
}

// One operand's loader state: which rows / k-rows this thread fetches and where they land in LDS.
template <int ROWS, int NV, int THREADS, bool BF16>
struct Loader {
    static constexpr int EPC = BF16 ? 8 : 4;
    static constexpr int CM = ROWS / EPC;            // mn-chunks per k-row (mn-contiguous mode)
    const char *base;                                // operand base for this (tuple, batch, tile)
    int64_t row_off[NV];                             // k-contiguous mode: element offset of each fetched row
    int64_t mn_off;                                  // mn-contiguous mode: element offset of the chunk start
    bool kcontig;
    uint4 reg[NV];

    // gsel: 0 -> K strides of X (s0), 1 -> K strides of Y (s1)
    __device__ __forceinline__ void init(const void *ptr, int64_t base_off, const DimList &grp, int64_t first, int64_t extent,
                                         bool kc, int tid)
    {
        kcontig = kc;
        base = (const char *)ptr + base_off * (BF16 ? 2 : 4);
        if (kc) {
#pragma unroll
            for (int i = 0; i < NV; i++) {
                int64_t r = first + (tid >> 3) + i * (THREADS / 8);
                r = r < extent ? r : extent - 1;                 // clamp: rows past the edge are never stored
                int64_t o0, o1;
                decode_group(grp, r, o0, o1);
                row_off[i] = o0;
            }
            mn_off = 0;
        } else {
            int64_t m = first + (int64_t)(tid % CM) * EPC;
            m = m + EPC <= extent ? m : extent - EPC;            // extent is a multiple of EPC (checked on the host)
            int64_t o0, o1;
            decode_group(grp, m, o0, o1);
            mn_off = o0;
#pragma unroll
            for (int i = 0; i < NV; i++) row_off[i] = 0;
        }
    }

    // Issues the global loads of the stage starting at k0.  which: 0 = X strides of K, 1 = Y strides.
    __device__ __forceinline__ void fetch(const DimList &kgrp, int which, int64_t k0, int64_t K, int tid)
    {
        if (kcontig) {
            const int64_t k = k0 + (tid & 7) * EPC;
            int64_t o0, o1;
            decode_group(kgrp, k < K ? k : 0, o0, o1);
            const int64_t ko = which ? o1 : o0;
#pragma unroll
            for (int i = 0; i < NV; i++) {
                if (k < K) reg[i] = *(const uint4 *)(base + (row_off[i] + ko) * (BF16 ? 2 : 4));
                else reg[i] = make_uint4(0, 0, 0, 0);
            }
        } else {
            const int64_t kfirst = k0 + (int64_t)(tid / CM) * NV;
#pragma unroll
            for (int i = 0; i < NV; i++) {
                const int64_t k = kfirst + i;
                int64_t o0, o1;
                decode_group(kgrp, k < K ? k : 0, o0, o1);
                const int64_t ko = which ? o1 : o0;
                if (k < K) reg[i] = *(const uint4 *)(base + (mn_off + ko) * (BF16 ? 2 : 4));
                else reg[i] = make_uint4(0, 0, 0, 0);
            }
        }
    }

    __device__ __forceinline__ void commit(char *lds_tile, int tid) const
    {
        if (kcontig) {
#pragma unroll
            for (int i = 0; i < NV; i++) {
                const int row = (tid >> 3) + i * (THREADS / 8);
                *(uint4 *)(lds_tile + lds_off(row, tid & 7)) = reg[i];
            }
        } else {
            transpose_store<NV, BF16>(reg, lds_tile, (tid % CM) * EPC, (tid / CM) * NV);
        }
    }
};

template <typename C>
__global__ __launch_bounds__(C::THREADS) void k_contract(const ContractParams p)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / C::WAVES_N, wn = wave % C::WAVES_N;

    // ---- workgroup -> (tuple, batch, tile); consecutive logical ids stay on one XCD -----------------
    const int64_t total = (int64_t)gridDim.x;
    int64_t logical;
    {
        const int64_t per = total / 8, rem = total % 8;
        const int64_t x = blockIdx.x % 8, j = blockIdx.x / 8;
        logical = x * per + (x < rem ? x : rem) + j;
    }
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t tb = logical / tiles;
    const int tl = (int)(logical - tb * tiles);
    constexpr int GM = 8;                                    // tile rows walked together for L2 reuse
    const int span = GM * p.tiles_n;
    const int grp = tl / span, first_m = grp * GM;
    const int gsz = (p.tiles_m - first_m) < GM ? (p.tiles_m - first_m) : GM;
    const int tile_m = first_m + (tl - grp * span) % gsz;
    const int tile_n = (tl - grp * span) / gsz;
    const int64_t tuple = tb / p.n_batch, bidx = tb - tuple * p.n_batch;

    int64_t bx, by, bz, agg;
    decode_tuple(p.ts, tuple, bx, by, bz, agg);
    {
        uint32_t rem = (uint32_t)bidx;
        for (int i = p.batch.n - 1; i >= 0; i--) {
            uint32_t e = (uint32_t)p.batch.ext[i], q = rem / e, k = rem - q * e;
            rem = q;
            bx += (int64_t)k * p.batch.s0[i];
            by += (int64_t)k * p.batch.s1[i];
            bz += (int64_t)k * p.batch.s2[i];
        }
    }
    const int64_t m0 = (int64_t)tile_m * C::BM, n0 = (int64_t)tile_n * C::BN;

    Loader<C::BM, C::NVA, C::THREADS, C::BF16> la;
    Loader<C::BN, C::NVB, C::THREADS, C::BF16> lb;
    la.init(p.x, bx, p.m, m0, p.M, p.a_kcontig != 0, tid);
    lb.init(p.y, by, p.n, n0, p.N, p.b_kcontig != 0, tid);

    f32x16 acc[C::MT][C::NT];
#pragma unroll
    for (int i = 0; i < C::MT; i++)
#pragma unroll
        for (int j = 0; j < C::NT; j++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;

    const int64_t nk = (p.K + C::BK - 1) / C::BK;
    la.fetch(p.k, 0, 0, p.K, tid);
    lb.fetch(p.k, 1, 0, p.K, tid);
    la.commit(smem, tid);
    lb.commit(smem + C::LDS_A, tid);
    __syncthreads();

    const int lrow = lane & 31, lhalf = lane >> 5;
    for (int64_t kt = 0; kt < nk; kt++) {
        const int cur = (int)(kt & 1);
        const char *sa = smem + cur * (C::LDS_A + C::LDS_B);
        const char *sb = sa + C::LDS_A;
        if (kt + 1 < nk) {
            la.fetch(p.k, 0, (kt + 1) * C::BK, p.K, tid);
            lb.fetch(p.k, 1, (kt + 1) * C::BK, p.K, tid);
        }
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            uint4 a[C::MT], b[C::NT];
#pragma unroll
            for (int i = 0; i < C::MT; i++) a[i] = *(const uint4 *)(sa + lds_off(wm * C::WM + i * 32 + lrow, 2 * ks + lhalf));
#pragma unroll
            for (int j = 0; j < C::NT; j++) b[j] = *(const uint4 *)(sb + lds_off(wn * C::WN + j * 32 + lrow, 2 * ks + lhalf));
#pragma unroll
            for (int i = 0; i < C::MT; i++)
#pragma unroll
                for (int j = 0; j < C::NT; j++) {
                    if (C::BF16) {
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8 *)&a[i], *(const bf16x8 *)&b[j], acc[i][j], 0, 0, 0);
                    } else {
                        const float *fa = (const float *)&a[i];
                        const float *fb = (const float *)&b[j];
#pragma unroll
                        for (int q = 0; q < 4; q++) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[q], fb[q], acc[i][j], 0, 0, 0);
                    }
                }
        }
        if (kt + 1 < nk) {
            char *na = smem + (cur ^ 1) * (C::LDS_A + C::LDS_B);
            la.commit(na, tid);
            lb.commit(na + C::LDS_A, tid);
        }
        __syncthreads();
    }

    // ---- epilogue: lane holds column (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 tile ----
    char *zb = (char *)p.out.ptr + (p.out.slab_elems ? agg * p.out.slab_elems * 4 : 0);
    const bool out_bf16 = p.out.dtype == EG_BF16;
#pragma unroll
    for (int j = 0; j < C::NT; j++) {
        const int64_t n = n0 + wn * C::WN + j * 32 + lrow;
        if (n >= p.N) continue;
        int64_t oy_unused, zn;
        decode_group(p.n, n, oy_unused, zn);
#pragma unroll
        for (int i = 0; i < C::MT; i++) {
#pragma unroll
            for (int r = 0; r < 16; r++) {
                const int64_t m = m0 + wm * C::WM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                if (m >= p.M) continue;
                int64_t ox_unused, zm;
                decode_group(p.m, m, ox_unused, zm);
                const float val = p.alpha * acc[i][j][r];
                const int64_t off = bz + zm + zn;
                if (out_bf16) ((uint16_t *)zb)[off] = f32_to_bf16(val);
                else ((float *)zb)[off] = val;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// The same tiling for any other scalar function (x) and reduction (+) of Section 3 of the paper (squared
// difference with sum, absolute difference with max, ...): no matrix instruction fits, so the tile is worked
// on the vector ALU.  256 threads as a 16 x 16 grid, each thread an 8 x 8 block of the 128 x 128 tile with
// rows ty + 16 i and columns tx + 16 j (the 16 lanes that differ in tx read 16 consecutive LDS rows, which the
// swizzle spreads over all banks, and write consecutive columns).  Operands pass through the same loaders and
// the same LDS layout as above.  The reduction runs over exactly K values: zero-filled tail slots are skipped,
// since (x)(0, 0) need not be the identity of (+).
// ------------------------------------------------------------------------------------------------
template <typename C, int OT, int OP>
__global__ __launch_bounds__(C::THREADS, 2) void k_contract_alu(const ContractParams p)
{
    static_assert(C::BM == 128 && C::BN == 128 && C::THREADS == 256, "16 x 16 threads of 8 x 8 outputs");
    extern __shared__ __attribute__((aligned(16))) char smem[];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;

    const int64_t total = (int64_t)gridDim.x;
    int64_t logical;
    {
        const int64_t per = total / 8, rem = total % 8;
        const int64_t x = blockIdx.x % 8, j = blockIdx.x / 8;
        logical = x * per + (x < rem ? x : rem) + j;
    }
    const int64_t tiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t tb = logical / tiles;
    const int tl = (int)(logical - tb * tiles);
    const int tile_m = tl % p.tiles_m, tile_n = tl / p.tiles_m;
    const int64_t tuple = tb / p.n_batch, bidx = tb - tuple * p.n_batch;

    int64_t bx, by, bz, agg;
    decode_tuple(p.ts, tuple, bx, by, bz, agg);
    {
        uint32_t rem = (uint32_t)bidx;
        for (int i = p.batch.n - 1; i >= 0; i--) {
            uint32_t e = (uint32_t)p.batch.ext[i], q = rem / e, k = rem - q * e;
            rem = q;
            bx += (int64_t)k * p.batch.s0[i];
            by += (int64_t)k * p.batch.s1[i];
            bz += (int64_t)k * p.batch.s2[i];
        }
    }
    const int64_t m0 = (int64_t)tile_m * C::BM, n0 = (int64_t)tile_n * C::BN;

    Loader<C::BM, C::NVA, C::THREADS, C::BF16> la;
    Loader<C::BN, C::NVB, C::THREADS, C::BF16> lb;
    la.init(p.x, bx, p.m, m0, p.M, p.a_kcontig != 0, tid);
    lb.init(p.y, by, p.n, n0, p.N, p.b_kcontig != 0, tid);

    float acc[8][8];
    const float ident = oplus_identity(OP >= 0 ? OP : p.oplus);
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc[i][j] = ident;

    const int64_t nk = (p.K + C::BK - 1) / C::BK;

    // one 16-byte chunk (EPC consecutive k) of the thread's 8 rows and 8 columns; `valid` k of it count
    auto chunk = [&](const char *sa, const char *sb, int c, int valid) {
        uint4 a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; i++) a[i] = *(const uint4 *)(sa + lds_off(ty + 16 * i, c));
#pragma unroll
        for (int j = 0; j < 8; j++) b[j] = *(const uint4 *)(sb + lds_off(tx + 16 * j, c));
#pragma unroll
        for (int e = 0; e < C::EPC; e++) {
            if (e >= valid) break;
            float xs[8], ys[8];
#pragma unroll
            for (int i = 0; i < 8; i++) {
                const uint32_t wa = ((const uint32_t *)&a[i])[C::BF16 ? e >> 1 : e], wb = ((const uint32_t *)&b[i])[C::BF16 ? e >> 1 : e];
                xs[i] = C::BF16 ? __uint_as_float((e & 1) ? (wa & 0xffff0000u) : (wa << 16)) : __uint_as_float(wa);
                ys[i] = C::BF16 ? __uint_as_float((e & 1) ? (wb & 0xffff0000u) : (wb << 16)) : __uint_as_float(wb);
            }
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int j = 0; j < 8; j++) acc[i][j] = oplus_t<OP>(p.oplus, acc[i][j], otimes_t<OT, false>(p.otimes, xs[i], ys[j], p.alpha));
            __builtin_amdgcn_sched_barrier(0);       // one k at a time: unpacking all of a chunk ahead of its use costs registers
        }
    };

    // One LDS stage, no register prefetch: a stage is some ten microseconds of arithmetic per wave, the other
    // workgroups on the compute unit cover the loads, and the registers are needed for the 8 x 8 block.
    const char *sa = smem, *sb = smem + C::LDS_A;
    for (int64_t kt = 0; kt < nk; kt++) {
        la.fetch(p.k, 0, kt * C::BK, p.K, tid);
        lb.fetch(p.k, 1, kt * C::BK, p.K, tid);
        la.commit(smem, tid);
        lb.commit(smem + C::LDS_A, tid);
        __syncthreads();
        const int64_t left = p.K - kt * C::BK;
        if (left >= C::BK) {
#pragma unroll 1
            for (int c = 0; c < 8; c++) chunk(sa, sb, c, C::EPC);
        } else {
            for (int c = 0; c * C::EPC < left; c++) chunk(sa, sb, c, (int)(left - c * C::EPC < C::EPC ? left - c * C::EPC : C::EPC));
        }
        __syncthreads();
    }

    char *zb = (char *)p.out.ptr + (p.out.slab_elems ? agg * p.out.slab_elems * 4 : 0);
    const bool out_bf16 = p.out.dtype == EG_BF16;
    int64_t zn[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int64_t n = n0 + tx + 16 * j;
        int64_t unused;
        decode_group(p.n, n < p.N ? n : 0, unused, zn[j]);
    }
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const int64_t m = m0 + ty + 16 * i;
        if (m >= p.M) continue;
        int64_t unused, zm;
        decode_group(p.m, m, unused, zm);
#pragma unroll
        for (int j = 0; j < 8; j++) {
            if (n0 + tx + 16 * j >= p.N) continue;
            const int64_t off = bz + zm + zn[j];
            if (out_bf16) ((uint16_t *)zb)[off] = f32_to_bf16(acc[i][j]);
            else ((float *)zb)[off] = acc[i][j];
        }
    }
}

template <typename C, int OT, int OP>
static int launch_alu(ContractParams &p, void *stream)
{
    p.tiles_m = (int32_t)((p.M + C::BM - 1) / C::BM);
    p.tiles_n = (int32_t)((p.N + C::BN - 1) / C::BN);
    const int64_t wgs = p.n_tuples * p.n_batch * p.tiles_m * p.tiles_n;
    if (wgs < 1 || wgs >= (1ll << 31)) return fail(EG_ERR_LIMIT, "contraction needs %lld workgroups", (long long)wgs);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)k_contract_alu<C, OT, OP>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_A + C::LDS_B) != hipSuccess)
            return fail(EG_ERR_HIP, "cannot reserve %d bytes of LDS", C::LDS_A + C::LDS_B);
        attr_set = true;
    }
    EG_LAUNCH((k_contract_alu<C, OT, OP>), dim3((unsigned)wgs), dim3(C::THREADS), C::LDS_A + C::LDS_B, (hipStream_t)stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "k_contract_alu launch failed: %s", hipGetErrorString(e));
    return EG_OK;
}

template <typename C>
static int launch_alu_ops(ContractParams &p, void *stream)
{
    // the paper's two examples are compiled in; any other pair reads its operators at run time
    if (p.otimes == EG_SQDIFF && p.oplus == EG_AGG_SUM) return launch_alu<C, EG_SQDIFF, EG_AGG_SUM>(p, stream);
    if (p.otimes == EG_ABSDIFF && p.oplus == EG_AGG_MAX) return launch_alu<C, EG_ABSDIFF, EG_AGG_MAX>(p, stream);
    return launch_alu<C, -1, -1>(p, stream);
}

template <typename C>
static int launch_cfg(ContractParams &p, void *stream)
{
    p.tiles_m = (int32_t)((p.M + C::BM - 1) / C::BM);
    p.tiles_n = (int32_t)((p.N + C::BN - 1) / C::BN);
    const int64_t wgs = p.n_tuples * p.n_batch * p.tiles_m * p.tiles_n;
    if (wgs < 1 || wgs >= (1ll << 31)) return fail(EG_ERR_LIMIT, "contraction needs %lld workgroups", (long long)wgs);
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute((const void *)k_contract<C>, hipFuncAttributeMaxDynamicSharedMemorySize, C::LDS_BYTES) != hipSuccess)
            return fail(EG_ERR_HIP, "cannot reserve %d bytes of LDS", C::LDS_BYTES);
        attr_set = true;
    }
    EG_LAUNCH(k_contract<C>, dim3((unsigned)wgs), dim3(C::THREADS), C::LDS_BYTES, (hipStream_t)stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "k_contract launch failed: %s", hipGetErrorString(e));
    return EG_OK;
}

// Blocks with at least 128 rows or columns take the direct-to-LDS kernel when their layout allows; force_kernel
// (tr_set_contract_variant) forces one of the two.  A handful of small fp32 blocks (configuration 1: eight blocks of
// 128^3) is a latency chain of slow MFMAs on as many compute units, which 64 x 64 tiles of the register-staged kernel
// spread over four times as many.  (Skinny products included: with 8192 x 4096 x 32..96 the half-empty tiles of that
// kernel still finish in 0.045 ms against 0.105-0.124 ms here.)
bool contract_takes_dma(const ContractParams &p)
{
    if (p.otimes != EG_MUL || p.oplus != EG_AGG_SUM) return false;
    const int64_t tiles128 = p.n_tuples * p.n_batch * ((p.M + 127) / 128) * ((p.N + 127) / 128);
    const bool tiny_f32 = p.in_dtype == EG_F32 && tiles128 <= 64;
    const bool want_dma = p.force_kernel ? p.force_kernel == 2 : ((p.M >= 128 || p.N >= 128) && !tiny_f32);
    return want_dma && contract_dma_eligible(p);
}

int launch_contract(ContractParams &p, void *stream)
{
    // what the kernel assumes, re-checked here so that a wrong table can never reach the device
    if (!p.x || !p.y || !p.out.ptr) return fail(EG_ERR_NULL, "contraction: NULL operand");
    if (p.m.n < 1 || p.n.n < 1 || p.k.n < 1 || p.M < 1 || p.N < 1 || p.K < 1 || p.n_batch < 1 || p.n_tuples < 1)
        return fail(EG_ERR_LIMIT, "contraction: empty role group");
    const int epc = p.in_dtype == EG_BF16 ? 8 : 4;
    const bool ok_a = p.a_kcontig ? (p.k.s0[p.k.n - 1] == 1 && p.k.ext[p.k.n - 1] % epc == 0)
                                  : (p.m.s0[p.m.n - 1] == 1 && p.m.ext[p.m.n - 1] % epc == 0);
    const bool ok_b = p.b_kcontig ? (p.k.s1[p.k.n - 1] == 1 && p.k.ext[p.k.n - 1] % epc == 0)
                                  : (p.n.s0[p.n.n - 1] == 1 && p.n.ext[p.n.n - 1] % epc == 0);
    if (!ok_a || !ok_b) return fail(EG_ERR_LIMIT, "contraction: operand is not vectorisable along its contiguous label");
    if (((uintptr_t)p.x & 15) || ((uintptr_t)p.y & 15)) return fail(EG_ERR_LIMIT, "contraction: operands must be 16-byte aligned");
    if (p.otimes != EG_MUL || p.oplus != EG_AGG_SUM) {
        if (p.otimes < EG_MUL || p.otimes > EG_SILU_MUL) return fail(EG_ERR_BAD_OP, "contraction: scalar function %d is not binary", p.otimes);
        if (p.in_dtype == EG_BF16) return launch_alu_ops<Cfg<128, 128, 64, 64, true>>(p, stream);
        return launch_alu_ops<Cfg<128, 128, 64, 64, false>>(p, stream);
    }
    const int64_t tiles128 = p.n_tuples * p.n_batch * ((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (contract_takes_dma(p)) return launch_contract_dma(p, stream);
    if (tiles128 <= 64) {
        if (p.in_dtype == EG_BF16) return launch_cfg<Cfg<64, 64, 32, 32, true>>(p, stream);
        return launch_cfg<Cfg<64, 64, 32, 32, false>>(p, stream);
    }
    if (p.in_dtype == EG_BF16) return launch_cfg<Cfg<128, 128, 64, 64, true>>(p, stream);
    // fp32 shapes the direct-to-LDS kernel cannot take: 256 x 256 tiles (eight waves of 128 x 64) once there are enough
    // of them to occupy half the chip (measured 98-113 TFLOP/s on 4096^3 and 8192^3 against 81-101 with 128 x 128 tiles)
    const int64_t tiles256 = p.n_tuples * p.n_batch * ((p.M + 255) / 256) * ((p.N + 255) / 256);
    if (tiles256 >= 128) return launch_cfg<Cfg<256, 256, 128, 64, false>>(p, stream);
    return launch_cfg<Cfg<128, 128, 64, 64, false>>(p, stream);
}

}  // namespace eg
