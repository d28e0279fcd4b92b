// Block contraction (bf16 or fp32 operands, fp32 accumulation) with direct global->LDS staging, no register round trip.
//
// Same operation as k_contract.hip (the per-block kernel K of Section 4.3 of the paper for (x) = multiply,
// (+) = sum, all tuples of the join in one launch), specialised for blocks of at least 128 x 128:
//   * 256 x 256 output tiles, 8 waves per workgroup (two per SIMD), each owning a 128x64 patch = 4x2 MFMA 32x32 tiles;
//     or 256 x 128 tiles with 4 waves of the same 128x64 patch, stages half as deep and two workgroups per compute unit,
//     so that one workgroup's epilogue, addressing and first loads run under the other's MFMAs;
//     or 128 x 128 tiles with 4 waves and two workgroups per compute unit when large tiles would leave the chip idle;
//   * persistent workgroups, each walking over its share of the output tiles;
//   * every 16-byte chunk of both operand tiles travels global memory -> LDS directly; the chunk a lane
//     fetches is chosen so that the contiguous 1 KiB an instruction deposits is already the swizzled layout;
//   * a stage is 128 (or 64) bytes of k per tile row (64 or 32 k of bf16, 32 k of fp32) and four (two) k-steps: one
//     32x32x16 bf16 MFMA per 32x32 tile and step, or four 32x32x2 fp32 MFMAs on the four k a 16-byte chunk brings;
//   * an operand contiguous along K sits in LDS as [row][128 bytes of k] and is read with 16-byte reads; an operand
//     contiguous along M or N sits as [k][TS mn] and is read with the 16-bit transposing LDS read (bf16), which
//     hands every lane four consecutive k for its own column, or with four 4-byte reads (fp32);
//   * two LDS stages: the loads of stage t+1 are in flight while the MFMAs of stage t run.
//   * the loads are buffer loads with a 2 GiB descriptor: a lane whose chunk lies beyond K in the last,
//     partial stage is given an offset outside the descriptor, fetches nothing and deposits zeros.
// Several K labels: every run of the innermost one starts a stage of its own (a run of 96 k is a full stage and
// a half-filled one), so a stage never straddles two runs.
// Requirements (checked on the host): along a K-contiguous operand runs are whole 16-byte chunks on chunk boundaries;
// byte offsets within a tile (256 rows, 64 k-rows) fit 31 bits and rows do not lie before their tile's first row.
// Anything else goes to the register-staged kernel.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "eg_device.h"

namespace eg {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

namespace dma {

// Element type: bf16 (F32 = false) or fp32.  A stage holds 128 bytes of k per row: 64 k of bf16, 32 k of fp32, and is
// four k-steps either way (one 32x32x16 bf16 MFMA, or four 32x32x2 fp32 MFMAs on the four k a 16-byte chunk brings).
template <bool F32> struct Elem {
    static constexpr int ES = F32 ? 4 : 2;         // bytes per element
    static constexpr int EPC = 16 / ES;            // elements per 16-byte chunk
};

#define EG_LDS(p) ((__attribute__((address_space(3))) void *)(p))
#define EG_GLB(p) ((const __attribute__((address_space(1))) void *)(p))

__device__ __forceinline__ void decode_group2(const DimList &g, int64_t idx, int64_t &o0, int64_t &o1)
{
    o0 = o1 = 0;
    if (g.n == 1) { o0 = idx * g.s0[0]; o1 = idx * g.s1[0]; return; }
    uint32_t rem = (uint32_t)idx;
    for (int i = g.n - 1; i >= 0; i--) {
        uint32_t e = (uint32_t)g.ext[i], q = rem / e, k = rem - q * e;
        rem = q;
        o0 += (int64_t)k * g.s0[i];
        o1 += (int64_t)k * g.s1[i];
    }
}

// Per-lane source offsets (bytes, relative to the first row of the operand's tile: `origin` is that row's
// element offset in the block) of the chunks this lane fetches per stage (NW waves per workgroup, T rows or columns
// of this operand per tile, KB bytes of k per row and stage), without the k advance.
//   KC: a row holds CR = KB/16 chunks, so one 1 KiB instruction deposits RPI = 64/CR rows (8 for KB = 128, 16 for 64):
//       instruction i of wave w deposits rows (NW i+w)*RPI .. +RPI-1, lane -> row +lane/CR, physical chunk lane%CR,
//       logical chunk (lane%CR) ^ key(row), key = (row>>1)&7 for 128-byte rows, (row>>2)&3 for 64-byte rows: the 16 rows a
//       16-byte LDS read instruction touches in one pass then fall into 16 different 16-byte bank groups.
//   MC: a k-row holds CPR = T/8 chunks, so one instruction deposits KR = 64/CPR k-rows (2 for T = 256, 4 for
//       T = 128): instruction i of wave w deposits k-rows KR (NW i+w) .. +KR-1, lane -> k-row +lane/CPR,
//       physical chunk lane%CPR, logical chunk (lane%CPR) ^ 4*(krow%4), krow%4 = (KR w + lane/CPR)%4.
template <bool KC, int NW, int T, int KB, bool F32>
struct Src {
    static constexpr int ES = Elem<F32>::ES, EPC = Elem<F32>::EPC;
    static constexpr int LD = T * KB / 1024 / NW;         // direct loads of this operand per wave and stage
    static constexpr int CR = KB / 16, RPI = 64 / CR;     // chunks per row of a KC tile, rows per 1 KiB instruction
    static constexpr int CPR = T / EPC, KR = 64 / CPR;    // chunks per k-row of an MC tile, k-rows per 1 KiB instruction
    static_assert(LD >= 1 && LD * NW * 1024 == T * KB, "a stage of this operand is a whole number of 1 KiB instructions per wave");
    static_assert(KB == 128 || KB == 64, "rows of 128 or 64 bytes of k");
    static_assert((NW * KR) % 4 == 0, "the swizzle key of an MC chunk must not depend on the instruction index");
    uint32_t boff[LD];        // byte offset of the chunk instruction i fetches, relative to the stage's first k
    int kl;                   // k (within the stage) of chunk 0 of this lane; chunk i sits at kl (KC) or kl + KR NW i (MC)

    __device__ __forceinline__ void init(const DimList &grp, int64_t first, int64_t extent, int64_t origin, int64_t k_inner_stride, int wave, int lane)
    {
        if (KC) {
            // LDS row of this lane's chunk is (NW i+wave)*RPI + lane/CR; its swizzle key does not depend on i
            const int key = KB == 128 ? ((wave * 4 + (lane >> 4)) & 7) : ((lane >> 4) & 3);
            const int lc = (lane % CR) ^ key;
            kl = lc * EPC;
#pragma unroll
            for (int i = 0; i < LD; i++) {
                int64_t r = first + (NW * i + wave) * RPI + lane / CR;
                r = r < extent ? r : extent - 1;
                int64_t o0, o1;
                decode_group2(grp, r, o0, o1);
                boff[i] = (uint32_t)((o0 - origin + lc * EPC) * ES);
            }
        } else {
            // bf16: chunks of four consecutive k-rows are XOR-ed apart for the transposing reads; fp32 fragments are read
            // with 4-byte reads of 32 consecutive columns, which need no swizzle
            const int kr4 = (KR * wave + lane / CPR) & 3;
            const int lc = F32 ? lane % CPR : (lane % CPR) ^ (4 * kr4);
            int64_t m = first + lc * EPC;
            m = m + EPC <= extent ? m : extent - EPC;
            int64_t o0, o1;
            decode_group2(grp, m, o0, o1);
            kl = KR * wave + lane / CPR;
#pragma unroll
            for (int i = 0; i < LD; i++)
                boff[i] = (uint32_t)((o0 - origin + (KR * NW * i + kl) * k_inner_stride) * ES);
        }
    }
    // offset handed to load i of a stage whose valid k are kmin .. krem-1: beyond the descriptor when the chunk's k is outside
    // (past the end of the reduction, or, in a tile's first stage, before its start)
    __device__ __forceinline__ uint32_t voff(int i, int krem, int kmin) const
    {
        const int k = KC ? kl : kl + KR * NW * i;
        return (uint32_t)(k - kmin) < (uint32_t)(krem - kmin) ? boff[i] : 0x80000000u;
    }
};

// LDS byte address of the fragment chunk lane `lane` feeds to the MFMA for 32-row tile `t32` (rows t32*32..+31
// of the wave's 128) at k-step ks (16 k per step).  KC layout: one 16-byte read.
template <int KB>
__device__ __forceinline__ int kc_frag_off(int row, int ks, int lane)
{
    const int lc = 2 * ks + (lane >> 5);
    const int key = KB == 128 ? (row >> 1) & 7 : (row >> 2) & 3;
    return row * KB + ((lc ^ key) << 4);                    // 16 consecutive rows hit 16 distinct 16-byte bank groups
}

// MC layout: two transposing 8-byte reads (k = 8*(lane/32) + 0..3 and +4..7 of the k-step); TS: columns of the operand's tile.
template <int TS>
__device__ __forceinline__ int mc_frag_off(int col0, int ks, int lane, int second)
{
    const int s = lane & 15;
    const int kr = 16 * ks + 8 * (lane >> 5) + (s >> 2) + 4 * second;
    const int n = col0 + 16 * ((lane >> 4) & 1) + 4 * (s & 3);
    const int pc = (n >> 3) ^ (4 * (s >> 2));
    return kr * (TS * 2) + (pc << 4) + ((n & 7) << 1);
}

// Fragments of one k-step (16 k of bf16, 8 k of fp32): RT 32-row A fragments and NT 32-column B fragments of this wave
// (row0, col0: first row / column of the wave's patch inside the tile).  A fragment is 16 bytes per lane: eight bf16
// (k = 8 * (lane / 32) + 0..7 of the step) or four fp32 (k = 4 * (lane / 32) + 0..3).
template <bool KC, int TS, int KB, bool F32>
__device__ __forceinline__ u32x4 load_frag(const char *l, int first, int ks, int lane)
{
    if (KC) return *(const u32x4 *)(l + kc_frag_off<KB>(first + (lane & 31), ks, lane));
    if (F32) {
        const char *q = l + (8 * ks + 4 * (lane >> 5)) * (TS * 4) + (first + (lane & 31)) * 4;
        u32x4 v;
        v.x = *(const uint32_t *)q; v.y = *(const uint32_t *)(q + TS * 4); v.z = *(const uint32_t *)(q + 2 * TS * 4); v.w = *(const uint32_t *)(q + 3 * TS * 4);
        return v;
    }
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)EG_LDS(l + mc_frag_off<TS>(first, ks, lane, 0)));
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) short4v *)EG_LDS(l + mc_frag_off<TS>(first, ks, lane, 1)));
    u32x4 v;
    short4v *dst = (short4v *)&v;
    dst[0] = lo; dst[1] = hi;
    return v;
}

template <bool A_KC, bool B_KC, int RT, int NT, int TM, int TN, int KB, bool F32>
__device__ __forceinline__ void load_frags(const char *la, const char *lb, int ks, u32x4 (&a)[RT], u32x4 (&b)[NT], int row0, int col0, int lane)
{
#pragma unroll
    for (int i = 0; i < RT; i++) a[i] = load_frag<A_KC, TM, KB, F32>(la, row0 + i * 32, ks, lane);
#pragma unroll
    for (int j = 0; j < NT; j++) b[j] = load_frag<B_KC, TN, KB, F32>(lb, col0 + j * 32, ks, lane);
}

// One 32x32 tile's share of a k-step.
template <bool F32>
__device__ __forceinline__ void mma(const u32x4 &a, const u32x4 &b, f32x16 &acc)
{
    if (F32) {
        // the elements are copied out first: a bit cast applied directly to an element of a vector reference read element 0 every time
        const uint32_t a0 = a.x, a1 = a.y, a2 = a.z, a3 = a.w, b0 = b.x, b1 = b.y, b2 = b.z, b3 = b.w;
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a0), __uint_as_float(b0), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a1), __uint_as_float(b1), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a2), __uint_as_float(b2), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a3), __uint_as_float(b3), acc, 0, 0, 0);
    } else {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
    }
}

// MFMAs of one k-step for rows [I0, I1) of this wave's RT x NT grid of 32x32 tiles.
template <int I0, int I1, int RT, int NT, bool F32>
__device__ __forceinline__ void mfma_rows(const u32x4 (&a)[RT], const u32x4 (&b)[NT], f32x16 (&acc)[RT][NT])
{
#pragma unroll
    for (int i = I0; i < I1; i++)
#pragma unroll
        for (int j = 0; j < NT; j++) mma<F32>(a[i], b[j], acc[i][j]);
}

// What is uniform over a workgroup about one output tile.
struct TileInfo {
    int64_t m0, n0;          // first row / column of the tile inside the block
    const char *xb, *yb;     // X and Y at the tuple's blocks, the batch entry and the tile's first row / column
    int64_t ox0, oy0;        // element offsets of that first row / column inside the block (what lane offsets are relative to)
    int64_t bz, agg;         // Z element offset of the tuple's block and batch entry; aggIdx of the tuple
    int64_t slab_tile;       // with tile-ordered partial slabs: the tile's place in its slab
};

// Output tiles are TM x TN; the NW waves of a workgroup form a 2 x NW/2 grid of patches; a stage holds KB bytes of k per row.
//   256 x 256, KB = 128, NW = 8: two waves per SIMD, each owning 128 x 64; one wave's MFMAs cover the other's LDS reads
//       and barrier waits.  One workgroup per compute unit (154 KiB of LDS): every tile's addressing, first loads and
//       epilogue run with the matrix pipes idle, which is what short reductions consist of.
//   256 x 128, KB = 64, NW = 4: the same 128 x 64 patch per wave (the same LDS reads per MFMA), stages half as deep, 64 KiB
//       of LDS: two workgroups per compute unit, not in step with each other, so one's per-tile phases and barrier waits
//       run under the other's MFMAs.
//   256 x 256, KB = 128, NW = 4: one wave per SIMD, each owning 128 x 128 (two thirds of the LDS read traffic, nothing to
//       cover a wave's own waits); kept for comparison.
//   128 x 128, KB = 128, NW = 4: patches of 64 x 64, 78 KiB of LDS, two workgroups per compute unit.  For launches with too
//       few larger tiles to fill the chip.
//
// The kernel is persistent: the workgroups of a compute unit walk over their share of the tiles.  While a tile's
// epilogue runs, the first two stages of the workgroup's next tile are already on their way into LDS, and the
// next tile's addressing was worked out while the current tile waited for its own first stage.
// LDS of one workgroup: the stages, two sets of Z offset tables, the waves' epilogue staging rows
// (with three stages the staging rows lie in the third stage's buffer, which is free while an epilogue runs)
constexpr int lds_bytes(int TM, int TN, int KB, int NW, int NS)
{
    return NS * (TM + TN) * KB + 2 * (TM + TN) * 8 + (NS == 2 ? NW * 8 * (32 * (TN / (NW / 2) / 32) * 4 + 32) : 0);
}

// NS: LDS stages (2 or 3); REM: the stage count modulo NS.
template <int TM, int TN, int KB, int NS, int NW, bool A_KC, bool B_KC, int REM, bool F32>
__global__ __launch_bounds__(NW * 64, 2 * lds_bytes(TM, TN, KB, NW, NS) <= 160 * 1024 ? 2 : 1) void k_contract_dma(const ContractParams p)
{
    constexpr int ES = Elem<F32>::ES, EPC = Elem<F32>::EPC, BK = KB / ES;
    constexpr int KS = KB / 32;                       // k-steps per stage (32 bytes of k each)
    constexpr int WN = NW / 2;                        // waves side by side
    constexpr int RT = TM / 64, NT = TN / WN / 32;    // 32x32 MFMA tiles per wave: RT down, NT across
    constexpr int LDA = TM * KB / 1024 / NW, LDB = TN * KB / 1024 / NW, NLD = LDA + LDB;   // direct loads per wave and stage
    constexpr int TILE_BYTES = TM * KB;               // X's tile of one stage: KB bytes of k per row; Y's follows it
    constexpr int STAGE_BYTES = (TM + TN) * KB;
    constexpr int TBL = (TM + TN) * 8;                // one set of Z offset tables (TM rows, TN columns)
    static_assert(KS == 4 || KS == 2, "a stage is four or two k-steps");
    constexpr int CW = 32 * NT, PITCH = CW * 4 + 32, WBUF = 8 * PITCH;   // epilogue staging: 8 rows of a wave's patch
    // Separate LDS objects for the two stages and for the epilogue: the compiler can then tell that the fragment
    // reads of one stage, or the epilogue's staging, never alias the direct loads in flight into another object,
    // and does not wait for them.
    __shared__ __attribute__((aligned(1024))) char lds0[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds1[STAGE_BYTES];
    __shared__ __attribute__((aligned(1024))) char lds2[NS == 3 ? STAGE_BYTES : 16];
    __shared__ __attribute__((aligned(16))) char ldsx[2 * TBL + (NS == 2 ? NW * WBUF : 0)];    // two sets of Z offset tables (+ staging)
    static_assert(NS == 2 || (NS == 3 && KS == 2 && NW * WBUF <= STAGE_BYTES), "three stages: half-depth stages, staging rows fit one of them");
    static_assert(REM >= 0 && REM < NS, "REM is the stage count modulo NS");
    static_assert(NS * STAGE_BYTES + 2 * TBL + (NS == 2 ? NW * WBUF : 0) == lds_bytes(TM, TN, KB, NW, NS), "lds_bytes() is what decides the workgroups per compute unit");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int row0 = wm * (32 * RT), col0 = wn * (32 * NT);

    // ---- this workgroup's tiles: logical ids first, first + stride, ...; concurrent ids share an XCD ----
    const uint32_t total = (uint32_t)p.total_tiles, G = gridDim.x;
    uint32_t first, stride, count;
    if ((G & 7) == 0) {
        const uint32_t per = total / 8, rem = total % 8, x = blockIdx.x % 8, j = blockIdx.x / 8;
        const uint32_t nx = per + (x < rem ? 1 : 0);
        stride = G / 8;
        first = x * per + (x < rem ? x : rem) + j;
        count = j < nx ? (nx - j + stride - 1) / stride : 0;
    } else {
        stride = G;
        first = blockIdx.x;
        count = first < total ? (total - first + G - 1) / G : 0;
    }
    if (count == 0) return;

    auto uniform_ptr = [](const char *q) {            // the buffer descriptors must live in scalar registers
        const uint64_t v = (uint64_t)q;
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
        return (const char *)(((uint64_t)hi << 32) | lo);
    };
    // logical id -> (tuple, batch entry, tile); tiles are walked in groups of 8 tile rows
    auto tile_info = [&](uint32_t logical, TileInfo &t) {
        const uint32_t tiles = (uint32_t)p.tiles_m * (uint32_t)p.tiles_n;
        const uint32_t tb = logical / tiles, tl = logical - tb * tiles;
        constexpr uint32_t GM = 8;
        const uint32_t span = GM * (uint32_t)p.tiles_n;
        const uint32_t grp = tl / span, first_m = grp * GM;
        const uint32_t gsz = ((uint32_t)p.tiles_m - first_m) < GM ? ((uint32_t)p.tiles_m - first_m) : GM;
        const uint32_t tile_m = first_m + (tl - grp * span) % gsz;
        const uint32_t tile_n = (tl - grp * span) / gsz;
        const uint32_t nb = (uint32_t)p.n_batch, tuple = tb / nb, bidx = tb - tuple * nb;
        int64_t bx, by, bz, agg;
        decode_tuple(p.ts, tuple, bx, by, bz, agg);
        uint32_t rem = bidx;
        for (int i = p.batch.n - 1; i >= 0; i--) {
            uint32_t e = (uint32_t)p.batch.ext[i], q = rem / e, k = rem - q * e;
            rem = q;
            bx += (int64_t)k * p.batch.s0[i];
            by += (int64_t)k * p.batch.s1[i];
            bz += (int64_t)k * p.batch.s2[i];
        }
        t.m0 = (int64_t)tile_m * TM;
        t.n0 = (int64_t)tile_n * TN;
        // lane offsets are 32 bits and count from the tile's first row (an operand contiguous along M or N reads whole
        // 8-element chunks, so near the block's edge its first chunk may start up to 7 elements before the tile)
        int64_t unused;
        const int64_t fm = A_KC || t.m0 + EPC <= p.M ? t.m0 : p.M - EPC, fn = B_KC || t.n0 + EPC <= p.N ? t.n0 : p.N - EPC;
        decode_group2(p.m, fm, t.ox0, unused);
        decode_group2(p.n, fn, t.oy0, unused);
        t.xb = uniform_ptr((const char *)p.x + (bx + t.ox0) * ES);
        t.yb = uniform_ptr((const char *)p.y + (by + t.oy0) * ES);
        t.bz = bz;
        t.agg = agg;
        t.slab_tile = p.tile_order ? ((tuple_group(p.ts, tuple) * nb + bidx) * (int64_t)p.tiles_m + tile_m) * (int64_t)p.tiles_n + tile_n : 0;
    };
    const int kin = p.k.n - 1;                        // innermost K label: every stage lies inside one run of it
    const int64_t run = p.k.n == 1 ? p.K : p.k.ext[kin];            // k of one run of the innermost K label
    const int64_t nk = p.k_stages;                    // stages per tile: every run starts a stage of its own

    TileInfo cur, nxt;
    Src<A_KC, NW, TM, KB, F32> sa;
    Src<B_KC, NW, TN, KB, F32> sb;
    const char *xb, *yb;                              // bases the direct loads currently work from

    // Uniform source pointers of consecutive stages, and how many k each has (a full stage, less at the end of a run of
    // the innermost K label, 0 past the end: every lane of its direct loads then deposits zeros without fetching).
    // Inside a run a stage lies one fixed step after the one before; where a run ends (several fused K labels) the
    // next stage starts the next run and its offsets are decoded afresh, so a stage never straddles two runs and the
    // main loop's scalar work per stage is two additions almost always.
    const int64_t dka = (int64_t)BK * p.k.s0[kin] * ES, dkb = (int64_t)BK * p.k.s1[kin] * ES;
    // With p.k_align (one K label, an operand contiguous along it whose rows all start at the same offset inside a 128-byte
    // line) a tile's stages are laid on that operand's lines: the first one starts `kskip` elements before the block's
    // first k, those elements are not fetched (zeros), and every later stage fetches whole lines instead of the halves of two.
    const char *ga_n, *gb_n;
    int64_t k_n, run_left;
    int kskip = 0, kmin_n = 0;
    auto first_stage = [&]() {
        k_n = -kskip;
        ga_n = xb - (int64_t)kskip * p.k.s0[kin] * ES;
        gb_n = yb - (int64_t)kskip * p.k.s1[kin] * ES;
        run_left = run + kskip;
        kmin_n = kskip;
    };
    auto next_stage = [&](const char *&ga, const char *&gb, int &krem, int &kmin) {
        ga = ga_n;
        gb = gb_n;
        krem = k_n >= p.K ? 0 : (run_left < BK ? (int)run_left : BK);
        kmin = kmin_n;
        kmin_n = 0;
        if (run_left > BK) {
            k_n += BK;
            run_left -= BK;
            ga_n += dka;
            gb_n += dkb;
        } else {
            k_n += run_left;
            run_left = run;
            if (k_n < p.K) {
                int64_t ka, kb;
                decode_group2(p.k, k_n, ka, kb);       // offset of the next run's first k in X and in Y
                ga_n = xb + ka * ES;
                gb_n = yb + kb * ES;
            }
        }
    };
    // direct load i (0..LDA-1: X tile, LDA..NLD-1: Y tile) of a stage into the LDS stage at `dst`: a 2 GiB buffer descriptor
    // on the uniform stage base + a 32-bit lane offset (in-block offsets are below 2^31; 2^31 itself means "no fetch, zeros")
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto dma = [&](int i, const char *ga, const char *gb, int krem, int kmin, char *dst) {
        if (i < LDA) {
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)ga, 0, (int)0x80000000u, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, EG_LDS(dst + (NW * i + wave_u) * 1024), 16, (int)sa.voff(i, krem, kmin), 0, 0, 0);
        } else {
            __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void *)gb, 0, (int)0x80000000u, 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, EG_LDS(dst + TILE_BYTES + (NW * (i - LDA) + wave_u) * 1024), 16, (int)sb.voff(i - LDA, krem, kmin), 0, 0, 0);
        }
    };
    // The same load written out by hand, for the loads that travel during an epilogue: the compiler keeps track of
    // direct loads it issued itself and would hold the epilogue's first LDS access until they have landed.  These
    // are waited for by the explicit vmcnt(0) and barrier at the head of the tile loop.  M0 (the LDS base of a
    // direct load) is put back, so the compiler's own picture of it stays right.
    auto dma_untracked = [&](int i, const char *ga, const char *gb, int krem, int kmin, char *dst) {
        const bool isa = i < LDA;
        const uint64_t base = (uint64_t)(isa ? ga : gb);
        u32x4 rs;
        rs.x = (uint32_t)base;
        rs.y = (uint32_t)(base >> 32) & 0xffffu;       // stride 0
        rs.z = 0x80000000u;
        rs.w = 0x00020000u;
        const uint32_t l = (uint32_t)(uintptr_t)EG_LDS(dst + (isa ? 0 : TILE_BYTES) + (NW * (isa ? i : i - LDA) + wave_u) * 1024);
        const uint32_t off = isa ? sa.voff(i, krem, kmin) : sb.voff(i - LDA, krem, kmin);
        uint32_t keep;
        asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                     : "=&s"(keep) : "s"(l), "v"(off), "s"(rs) : "memory");
    };
    auto issue = [&](const char *ga, const char *gb, int krem, int kmin, char *dst) {
#pragma unroll
        for (int i = 0; i < NLD; i++) dma_untracked(i, ga, gb, krem, kmin, dst);
    };
    const char *ga2, *gb2;
    int kr2, km2;
    // per-lane addressing of tile t, then its first two stages on their way (both LDS stages must be free)
    auto start_tile = [&](const TileInfo &t) {
        sa.init(p.m, t.m0, p.M, t.ox0, p.k.s0[kin], wave, lane);
        sb.init(p.n, t.n0, p.N, t.oy0, p.k.s1[kin], wave, lane);
        xb = uniform_ptr(t.xb);
        yb = uniform_ptr(t.yb);
        kskip = p.k_align ? (int)(((uint32_t)(uintptr_t)(p.k_align == 1 ? xb : yb) & 127u) / ES) : 0;
        first_stage();
        next_stage(ga2, gb2, kr2, km2);
        issue(ga2, gb2, kr2, km2, lds0);
        next_stage(ga2, gb2, kr2, km2);
        if (nk > 1) issue(ga2, gb2, kr2, km2, lds1);
    };

    // Software pipeline.  Fragment registers alternate between two sets (f0 = a0/b0, f1 = a1/b1).  Each k-step
    // issues its first NT MFMAs, then the LDS reads of the next k-step, then its other 3 NT MFMAs, so the reads
    // return while the matrix pipe is busy.  The last k-step of a stage runs after the barrier, together with
    // the direct loads of the stage after next and the first fragment reads of the next stage.
    // sched_barrier pins this order against the compiler's own scheduling.
    f32x16 acc[RT][NT];
    u32x4 a0[RT], b0[NT], a1[RT], b1[NT];
#define EG_PIN() __builtin_amdgcn_sched_barrier(0)
#define EG_FRAGS(BUF, KSTEP, NA, NB) load_frags<A_KC, B_KC, RT, NT, TM, TN, KB, F32>(BUF, BUF + TILE_BYTES, KSTEP, NA, NB, row0, col0, lane)
#define EG_KSTEP(FA, FB, NA, NB, BUF, KS_NEXT)                                                    \
    mfma_rows<0, 1, RT, NT, F32>(FA, FB, acc); EG_PIN();                                                   \
    EG_FRAGS(BUF, KS_NEXT, NA, NB); EG_PIN();                                                      \
    mfma_rows<1, RT, RT, NT, F32>(FA, FB, acc); EG_PIN();
    // the direct loads of a stage are spread over the RT * NT MFMAs of a k-step: those that follow MFMA q
#define EG_DMA_AFTER(Q, C)                                                                        \
    if (has2) { _Pragma("unroll") for (int d = (Q) * NLD / (RT * NT); d < ((Q) + 1) * NLD / (RT * NT); d++) dma(d, ga2, gb2, kr2, km2, C); }
#define EG_STAGE_NEXT(C, O, HAS_NEXT2) /* one stage; its successor is already in flight into O */     \
    do {                                                                                          \
        mfma_rows<0, 1, RT, NT, F32>(a0, b0, acc); EG_PIN();                                               \
        const bool has2 = (HAS_NEXT2);                                                            \
        next_stage(ga2, gb2, kr2, km2);          /* scalar work rides under the MFMAs */               \
        EG_FRAGS(C, 1, a1, b1); EG_PIN();                                                         \
        mfma_rows<1, RT, RT, NT, F32>(a0, b0, acc); EG_PIN();                                               \
        if constexpr (KS == 4) {                                                                  \
            EG_KSTEP(a1, b1, a0, b0, C, 2)                                                        \
            EG_KSTEP(a0, b0, a1, b1, C, 3)                                                        \
        }                                                                                         \
        __builtin_amdgcn_s_waitcnt(0x0F70); /* vmcnt(0): this wave's deposits for O landed */     \
        __syncthreads();                    /* everybody's landed; everybody has left C */        \
        EG_PIN();                                                                                 \
        /* last k-step: the MFMAs carry the direct loads of the stage after next into C */        \
        _Pragma("unroll") for (int j = 0; j < NT; j++) {                                          \
            mma<F32>(a1[0], b1[j], acc[0][j]); EG_PIN();                                          \
            EG_DMA_AFTER(j, C)                                                                    \
            EG_PIN();                                                                             \
        }                                                                                         \
        EG_FRAGS(O, 0, a0, b0); EG_PIN();                                                         \
        _Pragma("unroll") for (int q = 0; q < (RT - 1) * NT; q++) {                               \
            mma<F32>(a1[1 + q / NT], b1[q % NT], acc[1 + q / NT][q % NT]); EG_PIN();              \
            EG_DMA_AFTER(NT + q, C)                                                               \
            EG_PIN();                                                                             \
        }                                                                                         \
    } while (0)

    // Three stages (two k-steps each): while stage s is computed, stage s+1 has landed or is landing and stage s+2 is in
    // flight; the loads of stage s+3 go into s's buffer once every wave has its last fragments of s in registers.  A load
    // has two full stages to arrive.  The wait before the barrier leaves the youngest stage's loads outstanding.
#define EG_STAGE3(C, O, HAS_NEXT2, HAS_NEXT3)                                                     \
    do {                                                                                          \
        mfma_rows<0, 1, RT, NT, F32>(a0, b0, acc); EG_PIN();                                               \
        const bool has2 = (HAS_NEXT3);      /* what EG_DMA_AFTER issues: stage s+3 into C */      \
        next_stage(ga2, gb2, kr2, km2);                                                                \
        EG_FRAGS(C, 1, a1, b1); EG_PIN();                                                         \
        mfma_rows<1, RT, RT, NT, F32>(a0, b0, acc); EG_PIN();                                               \
        /* vmcnt(NLD): stage s+1 has landed, stage s+2 may still travel; lgkmcnt(0): this wave's reads of C have returned. */ \
        /* A bare barrier: __syncthreads() would add a fence that waits for every outstanding load. */ \
        if (HAS_NEXT2) __builtin_amdgcn_s_waitcnt(0x0070 | (NLD & 15) | ((NLD >> 4) << 14));      \
        else __builtin_amdgcn_s_waitcnt(0x0070);                                                  \
        __builtin_amdgcn_s_barrier();                                                             \
        EG_PIN();                                                                                 \
        _Pragma("unroll") for (int j = 0; j < NT; j++) {                                          \
            mma<F32>(a1[0], b1[j], acc[0][j]); EG_PIN();                                          \
            EG_DMA_AFTER(j, C)                                                                    \
            EG_PIN();                                                                             \
        }                                                                                         \
        EG_FRAGS(O, 0, a0, b0); EG_PIN();                                                         \
        _Pragma("unroll") for (int q = 0; q < (RT - 1) * NT; q++) {                               \
            mma<F32>(a1[1 + q / NT], b1[q % NT], acc[1 + q / NT][q % NT]); EG_PIN();              \
            EG_DMA_AFTER(NT + q, C)                                                               \
            EG_PIN();                                                                             \
        }                                                                                         \
    } while (0)

    const bool out_bf16 = p.out.dtype == EG_BF16;

    tile_info(first, cur);
    start_tile(cur);
    for (uint32_t it = 0;; it++) {
        const bool more = it + 1 < count;
        // while the first stages travel: the next tile's uniform addressing and this tile's Z offset tables
        // (256 rows, 256 columns; two sets in turn, so a wave already in the next tile cannot disturb a slower one)
        if (more) tile_info(first + (it + 1) * stride, nxt);
        int64_t *zrow = (int64_t *)(ldsx + (it & 1) * TBL), *zcol = zrow + TM;
        if (!p.tile_order)                            // (tile-ordered partial slabs need no Z offsets)
        for (int e = tid; e < TM + TN; e += NW * 64) {
            int64_t unused, z;
            if (e < TM) {
                const int64_t m = cur.m0 + e;
                decode_group2(p.m, m < p.M ? m : 0, unused, z);
            } else {
                const int64_t n = cur.n0 + (e - TM);
                decode_group2(p.n, n < p.N ? n : 0, unused, z);
            }
            zrow[e] = z;
        }
#pragma unroll
        for (int i = 0; i < RT; i++)
#pragma unroll
            for (int j = 0; j < NT; j++)
#pragma unroll
                for (int r = 0; r < 16; r++) acc[i][j][r] = 0.f;
        __builtin_amdgcn_s_waitcnt(0x0F70);           // the first two stages (and the previous tile's stores) are done
        __syncthreads();
        if constexpr (NS == 3) {
            // the third buffer held the previous tile's staging rows until this barrier: its stage goes out now
            next_stage(ga2, gb2, kr2, km2);
            if (nk > 2) {
#pragma unroll
                for (int i = 0; i < NLD; i++) dma(i, ga2, gb2, kr2, km2, lds2);
            }
        }
        EG_FRAGS(lds0, 0, a0, b0);
        // Every stage, the last one included, runs the same straight-line code (the last one pays for one idle
        // barrier and a set of unused fragment reads): an MFMA under a branch inside the loop would make the
        // compiler shuffle the accumulator registers.  The stage count modulo the number of buffers is a template parameter.
        if constexpr (NS == 2) {
            if (REM) {
                EG_STAGE_NEXT(lds0, lds1, 2 < nk);
                for (int64_t st = 1; st < nk; st += 2) {
                    EG_STAGE_NEXT(lds1, lds0, st + 2 < nk);
                    EG_STAGE_NEXT(lds0, lds1, st + 3 < nk);
                }
            } else {
                for (int64_t st = 0; st < nk; st += 2) {
                    EG_STAGE_NEXT(lds0, lds1, st + 2 < nk);
                    EG_STAGE_NEXT(lds1, lds0, st + 3 < nk);
                }
            }
        } else {
            int64_t st = 0;
            for (; st + 3 <= nk; st += 3) {
                EG_STAGE3(lds0, lds1, st + 2 < nk, st + 3 < nk);
                EG_STAGE3(lds1, lds2, st + 3 < nk, st + 4 < nk);
                EG_STAGE3(lds2, lds0, st + 4 < nk, st + 5 < nk);
            }
            if constexpr (REM >= 1) EG_STAGE3(lds0, lds1, st + 2 < nk, false);
            if constexpr (REM == 2) EG_STAGE3(lds1, lds2, false, false);
        }
        __syncthreads();                              // every wave has left the stages
        // (three stages: the staging rows lie in a stage buffer the compiler has seen direct loads go into; all of those have
        // landed, and saying so here keeps it from waiting again, for the next tile's loads too, in front of the staging)
        if constexpr (NS == 3) __builtin_amdgcn_s_waitcnt(0x0F70);
        if (more) start_tile(nxt);                    // travels during the epilogue

        // ---- epilogue of the current tile -----------------------------------------------------------
        // lane holds column (lane % 32) and rows 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 tile
        char *zb = (char *)p.out.ptr + (p.out.slab_elems ? cur.agg * p.out.slab_elems * 4 : 0);
        // Everything per-lane below is derived from a lane id the compiler cannot see through, or it would work
        // out the addressing of all the unrolled stores once, before the tile loop, and keep it in scratch memory.
        int elane = lane;
        asm volatile("" : "+v"(elane));
        const int lrow = elane & 31, lhalf = elane >> 5;
        char *wbuf = (NS == 3 ? lds2 : ldsx + 2 * TBL) + wave_u * WBUF;   // this wave's staging rows
        const bool slab = p.out.slab_elems != 0;
        const int mrem = (int)(p.M - cur.m0 < TM ? p.M - cur.m0 : TM);     // rows / columns of the tile inside the block
        const int nrem = (int)(p.N - cur.n0 < TN ? p.N - cur.n0 : TN);
        if (p.tile_order) {
            // Partial slabs in tile order (the launcher set this only for whole tiles): every accumulator register group goes out
            // as it is, 16 bytes per lane and 1 KiB per instruction, no staging; the aggregation kernel undoes the layout.
            float *tb = (float *)zb + cur.slab_tile * (TM * TN) + (int64_t)wave_u * (RT * NT * 4 * 64 * 4);
#pragma unroll
            for (int i = 0; i < RT; i++)
#pragma unroll
                for (int j = 0; j < NT; j++)
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        const f32x4 val = {p.alpha * acc[i][j][4 * g], p.alpha * acc[i][j][4 * g + 1], p.alpha * acc[i][j][4 * g + 2], p.alpha * acc[i][j][4 * g + 3]};
                        __builtin_nontemporal_store(val, (f32x4 *)(tb + (((i * NT + j) * 4 + g) * 64 + elane) * 4));
                    }
        } else if (p.out_vec) {
            // Z is contiguous along the tile's columns: each wave stages 8 rows x CW columns of its patch at a time
            // in LDS (the row pitch leaves 32 bytes of padding, which keeps the two half-waves on different banks)
            // and writes them out as whole row segments, 16 bytes per lane.  LDS operations of one wave execute
            // in order, so no barrier is needed.
            // The 16 passes are software-pipelined: the stores of a pass are issued after the LDS writes and reads of
            // the next one, so a pass's LDS round trip is hidden behind the next pass's LDS traffic (the wave's LDS
            // operations stay in order, so the single staging buffer is enough).
            constexpr int LPR_F = CW / 4, RPI_F = 64 / LPR_F;     // fp32 out: lanes per row, rows per store instruction
            constexpr int LPR_B = CW / 8, RPI_B = 64 / LPR_B;     // bf16 out
            static_assert(RPI_F <= 8 && RPI_B <= 8, "a store instruction covers at most the 8 staged rows");
            constexpr int NV4 = CW / 32;                          // 16-byte LDS reads per lane and pass
            const int lc = out_bf16 ? elane % LPR_B : elane % LPR_F, lr = out_bf16 ? elane / LPR_B : elane / LPR_F;
            const int c = col0 + lc * (out_bf16 ? 8 : 4);         // first of this lane's 8 or 4 consecutive columns
            const int64_t zc = cur.bz + zcol[c];
            const bool cok = c < nrem;
            f32x4 rd[2][NV4];
            int64_t zr[2][NV4];
            auto write_pass = [&](int i, int q) {
#pragma unroll
                for (int j = 0; j < NT; j++)
#pragma unroll
                    for (int rr = 0; rr < 4; rr++)
                        *(float *)(wbuf + (4 * lhalf + rr) * PITCH + (j * 32 + lrow) * 4) = p.alpha * acc[i][j][4 * q + rr];
            };
            auto read_pass = [&](int i, int q, f32x4 (&v)[NV4], int64_t (&z)[NV4]) {
                if (!out_bf16) {
#pragma unroll
                    for (int h = 0; h < 8 / RPI_F; h++) {
                        const int row = RPI_F * h + lr;
                        v[h] = *(const f32x4 *)(wbuf + row * PITCH + lc * 16);
                        z[h] = zrow[row0 + i * 32 + 8 * q + row];
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < 8 / RPI_B; h++) {
                        const int row = RPI_B * h + lr;
                        v[2 * h] = *(const f32x4 *)(wbuf + row * PITCH + lc * 32);
                        v[2 * h + 1] = *(const f32x4 *)(wbuf + row * PITCH + lc * 32 + 16);
                        z[2 * h] = zrow[row0 + i * 32 + 8 * q + row];
                    }
                }
            };
            auto store_pass = [&](int i, int q, const f32x4 (&v)[NV4], const int64_t (&z)[NV4]) {
                if (!out_bf16) {
#pragma unroll
                    for (int h = 0; h < 8 / RPI_F; h++) {
                        const int rr = row0 + i * 32 + 8 * q + RPI_F * h + lr;
                        if (cok && rr < mrem) {
                            f32x4 *dst = (f32x4 *)((float *)zb + z[h] + zc);
                            const f32x4 val = v[h];
                            if (slab) __builtin_nontemporal_store(val, dst);   // partial slabs are read much later, by another kernel
                            else *dst = val;
                        }
                    }
                } else {
#pragma unroll
                    for (int h = 0; h < 8 / RPI_B; h++) {
                        const int rr = row0 + i * 32 + 8 * q + RPI_B * h + lr;
                        uint4 o;
                        o.x = pack_bf16x2(v[2 * h].x, v[2 * h].y); o.y = pack_bf16x2(v[2 * h].z, v[2 * h].w);
                        o.z = pack_bf16x2(v[2 * h + 1].x, v[2 * h + 1].y); o.w = pack_bf16x2(v[2 * h + 1].z, v[2 * h + 1].w);
                        if (cok && rr < mrem) *(uint4 *)((uint16_t *)zb + z[2 * h] + zc) = o;
                    }
                }
            };
#pragma unroll
            for (int ps = 0; ps < 4 * RT; ps++) {
                write_pass(ps >> 2, ps & 3);
                read_pass(ps >> 2, ps & 3, rd[ps & 1], zr[ps & 1]);
                __builtin_amdgcn_sched_barrier(0);
                if (ps > 0) store_pass((ps - 1) >> 2, (ps - 1) & 3, rd[(ps - 1) & 1], zr[(ps - 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
            store_pass(RT - 1, 3, rd[1], zr[1]);
        } else {
            int64_t zn[NT];
            bool nok[NT];
#pragma unroll
            for (int j = 0; j < NT; j++) {
                const int c = col0 + j * 32 + lrow;
                zn[j] = cur.bz + zcol[c];
                nok[j] = c < nrem;
            }
#pragma unroll
            for (int i = 0; i < RT; i++) {
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    const int rr = row0 + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                    if (rr < mrem) {
                        const int64_t zm = zrow[rr];
#pragma unroll
                        for (int j = 0; j < NT; j++) {
                            if (!nok[j]) continue;
                            const float val = p.alpha * acc[i][j][r];
                            const int64_t off = zm + zn[j];
                            if (out_bf16) ((uint16_t *)zb)[off] = f32_to_bf16(val);
                            else ((float *)zb)[off] = val;
                        }
                    }
                    asm volatile("" ::: "memory");     // keep the scheduler from hoisting all 64 row lookups at once
                }
            }
        }
        if (!more) break;
        cur = nxt;
    }
#undef EG_STAGE3
#undef EG_STAGE_NEXT
#undef EG_DMA_AFTER
#undef EG_KSTEP
#undef EG_FRAGS
#undef EG_PIN
}

template <int TM, int TN, int KB, int NS, int NW, bool A_KC, bool B_KC, int REM, bool F32>
static int launch_one(ContractParams &p, void *stream)
{
    EG_LAUNCH((k_contract_dma<TM, TN, KB, NS, NW, A_KC, B_KC, REM, F32>), dim3((unsigned)p.grid), dim3(NW * 64), 0, (hipStream_t)stream, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "k_contract_dma launch failed: %s", hipGetErrorString(e));
    return EG_OK;
}

template <int TM, int TN, int KB, int NS, int NW, bool A_KC, bool B_KC, bool F32>
static int launch_rem(ContractParams &p, void *stream)
{
    const int rem = (int)(p.k_stages % NS);
    if (rem == 0) return launch_one<TM, TN, KB, NS, NW, A_KC, B_KC, 0, F32>(p, stream);
    if (rem == 1) return launch_one<TM, TN, KB, NS, NW, A_KC, B_KC, 1, F32>(p, stream);
    if constexpr (NS == 3) return launch_one<TM, TN, KB, NS, NW, A_KC, B_KC, 2, F32>(p, stream);
    return fail(EG_ERR_LIMIT, "k_contract_dma: stage count");
}

template <int TM, int TN, int KB, int NS, int NW, bool F32>
static int launch_layout(ContractParams &p, void *stream)
{
    if (p.a_kcontig) return p.b_kcontig ? launch_rem<TM, TN, KB, NS, NW, true, true, F32>(p, stream) : launch_rem<TM, TN, KB, NS, NW, true, false, F32>(p, stream);
    return p.b_kcontig ? launch_rem<TM, TN, KB, NS, NW, false, true, F32>(p, stream) : launch_rem<TM, TN, KB, NS, NW, false, false, F32>(p, stream);
}

}  // namespace dma

bool contract_dma_eligible(const ContractParams &p)
{
    if (p.in_dtype != EG_BF16 && p.in_dtype != EG_F32) return false;
    const bool f32 = p.in_dtype == EG_F32;
    const int64_t es = f32 ? 4 : 2, epc = 16 / es, bk = 128 / es;
    if (p.m.n < 1 || p.n.n < 1 || p.k.n < 1) return false;
    // every run of the innermost K label starts a stage; along a K-contiguous operand 16-byte chunks must be whole and
    // aligned, so runs are whole chunks and start on chunk boundaries
    const int64_t run = p.k.n == 1 ? p.K : p.k.ext[p.k.n - 1];
    (void)bk;
    if (p.a_kcontig || p.b_kcontig) {
        if (run % epc) return false;
        for (int i = 0; i + 1 < p.k.n; i++)
            if ((p.a_kcontig && p.k.s0[i] % epc) || (p.b_kcontig && p.k.s1[i] % epc)) return false;
    }
    // Lane offsets count from the tile's first row and must stay below 2^31 bytes: rows of a tile must not lie before
    // its first row (strides nested, outermost first), and 256 rows plus the k-rows of a stage must span less.
    auto tile_span = [](const DimList &g) -> int64_t {            // largest offset of a row within 255 rows of another
        int64_t inner = 1, span = 0;
        for (int i = g.n - 1; i >= 0; i--) {
            if (g.s0[i] < 0) return -1;
            if (i + 1 < g.n && g.s0[i] < g.s0[i + 1] * g.ext[i + 1]) return -1;
            const int64_t steps = std::min<int64_t>(g.ext[i] - 1, 255 / inner + 1);
            span += steps * g.s0[i];
            inner *= g.ext[i];
        }
        return span;
    };
    const int kin = p.k.n - 1;
    const int64_t sx = tile_span(p.m), sy = tile_span(p.n);
    if (sx < 0 || sy < 0) return false;
    const int64_t lim = ((1ll << 31) - 256) / es;                           // elements
    if (sx + (p.a_kcontig ? 64 : 64 * std::max<int64_t>(p.k.s0[kin], 1)) >= lim) return false;
    if (sy + (p.b_kcontig ? 64 : 64 * std::max<int64_t>(p.k.s1[kin], 1)) >= lim) return false;
    if (p.a_kcontig ? p.k.s0[p.k.n - 1] != 1 : (p.m.s0[p.m.n - 1] != 1 || p.m.ext[p.m.n - 1] % epc)) return false;
    if (p.b_kcontig ? p.k.s1[p.k.n - 1] != 1 : (p.n.s0[p.n.n - 1] != 1 || p.n.ext[p.n.n - 1] % epc)) return false;
    if (!p.a_kcontig && p.M < epc) return false;
    if (!p.b_kcontig && p.N < epc) return false;
    if (((uintptr_t)p.x & 15) || ((uintptr_t)p.y & 15)) return false;
    return true;
}

// compute units of the current device, rounded down to whole XCD rounds (0: the device cannot be queried)
static int dma_cu_count()
{
    static int n_cu = 0;
    if (!n_cu) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 0;
        n_cu = prop.multiProcessorCount > 8 ? prop.multiProcessorCount / 8 * 8 : 8;
    }
    return n_cu;
}

void contract_dma_variant(const ContractParams &p, int &tm, int &tn, int &nw)
{
    const int n_cu = dma_cu_count();
    // Tile shape.  256 x 256, one workgroup per compute unit, is the fastest per flop on long reductions (fewest bytes into LDS per
    // flop, full 128-byte lines from operands contiguous along K).  256 x 128 with half-depth stages runs two workgroups per unit,
    // one's per-tile phases under the other's MFMAs; its main loop is a fifth slower (64-byte requests for operands contiguous
    // along K, a barrier every 16 MFMAs), so it is taken only where tiles are mostly per-tile work or where the wider tile would be
    // padding: reductions of up to 128 elements (config 4's scores: 0.42 -> 0.38 ms) and blocks whose last 256 columns are at most
    // half filled (config 4's P x V with 128 columns: 0.31 -> 0.30 ms).  128 x 128 tiles, two workgroups per unit, are taken
    // when they are all resident at once, i.e. when larger tiles would leave at least half of the compute units without work
    // (measured: 64 tiles of 256 x 256 ran 1.5-1.8x faster as 256 small ones; 160 of them 1.4x slower as 640 small ones, which
    // need a second round).
    const bool f32 = p.in_dtype == EG_F32;
    const int64_t tuples = p.n_tuples * p.n_batch;
    auto count = [&](int tm, int tn) { return tuples * ((p.M + tm - 1) / tm) * ((p.N + tn - 1) / tn); };
    const int64_t small = count(128, 128);
    const int64_t ntail = p.N % 256;
    if (small <= 2 * n_cu) tm = tn = 128;
    else if (!f32 && (p.K <= 128 || (ntail > 0 && ntail <= 128 && p.N < 1024))) { tm = 256; tn = 128; }
    else if (4 * count(256, 256) * 10 > small * 14) tm = tn = 128;
    else tm = tn = 256;
    if (p.force_tile_m && p.force_tile_n) { tm = p.force_tile_m; tn = p.force_tile_n; }   // tr_set_contract_variant: comparisons and tests
    if (f32 && tm != tn) tn = tm;
    nw = (tm == 256 && tn == 256 && (f32 || p.force_waves != 4)) ? 8 : 4;
}

int launch_contract_dma(ContractParams &p, void *stream)
{
    if (!p.x || !p.y || !p.out.ptr) return fail(EG_ERR_NULL, "contraction: NULL operand");
    if (!contract_dma_eligible(p)) return fail(EG_ERR_LIMIT, "contraction: shape not eligible for the direct-to-LDS kernel");
    const int n_cu = dma_cu_count();
    if (!n_cu) return fail(EG_ERR_HIP, "cannot query the device");
    const bool f32 = p.in_dtype == EG_F32;
    const int64_t tuples = p.n_tuples * p.n_batch;
    int tm, tn, nw;
    contract_dma_variant(p, tm, tn, nw);
    if (p.tile_order && (p.M % tm || p.N % tn || !p.out.slab_elems)) return fail(EG_ERR_LIMIT, "contraction: tile-ordered partial slabs need whole tiles");
    // the variant: stage depth and waves follow from the tile shape
    const int kb = (tm == 256 && tn == 128) ? 64 : 128;
    p.tiles_m = (int32_t)((p.M + tm - 1) / tm);
    p.tiles_n = (int32_t)((p.N + tn - 1) / tn);
    const int64_t wgs = tuples * p.tiles_m * p.tiles_n;
    if (wgs < 1 || wgs >= (1ll << 31)) return fail(EG_ERR_LIMIT, "contraction has %lld output tiles", (long long)wgs);
    // persistent workgroups: as many as fit the chip at once, a multiple of 8 so that every XCD gets the same number
    const int ns = kb == 64 ? 3 : 2;
    const int64_t resident = (2 * dma::lds_bytes(tm, tn, kb, nw, ns) <= 160 * 1024 ? 2 : 1) * (int64_t)n_cu;
    p.total_tiles = (int32_t)wgs;
    p.grid = (int32_t)(wgs < resident ? wgs : resident);
    // wide epilogue stores need Z contiguous along the innermost N label and every other Z offset a multiple of 8 elements
    bool vec = p.n.s1[p.n.n - 1] == 1 && p.n.ext[p.n.n - 1] % 8 == 0 && ((uintptr_t)p.out.ptr & 15) == 0 && p.out.slab_elems % 8 == 0;
    for (int i = 0; i < p.m.n; i++) vec = vec && p.m.s1[i] % 8 == 0;
    for (int i = 0; i + 1 < p.n.n; i++) vec = vec && p.n.s1[i] % 8 == 0;
    for (int i = 0; i < p.batch.n; i++) vec = vec && p.batch.s2[i] % 8 == 0;
    for (int l = 0; l < p.ts.n; l++) vec = vec && p.ts.step_z[l] % 8 == 0;
    p.out_vec = vec ? 1 : 0;
    // Stages per tile.  Where an operand is contiguous along the one K label and its blocks start inside a 128-byte line
    // (a slice of 1376 bf16: every other block starts 64 bytes into a line), stages that start at the block's first k fetch
    // two half lines per row and stage (config 4's down projection: 830 against 1030-1090 TFLOP/s with aligned slices).
    // k_align lays the stages on that operand's lines instead; the set of offsets the tuples' blocks can have decides how
    // many stages that takes, and a tile whose own offset needs one fewer runs an empty last stage.
    const int64_t es = f32 ? 4 : 2, bk = kb / es, run = p.k.n == 1 ? p.K : p.k.ext[p.k.n - 1];
    const int64_t stages0 = (p.K / run) * ((run + bk - 1) / bk);
    p.k_align = 0;
    p.k_stages = (int32_t)stages0;
    if (kb == 128 && p.k.n == 1 && stages0 >= 8) {
        // largest offset (in 16-byte chunks, 0..7) of a block's first row inside its line; -1: rows differ among themselves
        auto worst = [&](const void *base, int which) -> int {
            auto bytes = [&](int64_t elems) { return (uint64_t)(elems * es); };
            const DimList &rows = which == 0 ? p.m : p.n;
            for (int i = 0; i < rows.n; i++)
                if (rows.ext[i] > 1 && bytes(rows.s0[i]) % 128) return -1;
            for (int i = 0; i < p.batch.n; i++)
                if (p.batch.ext[i] > 1 && bytes(which == 0 ? p.batch.s0[i] : p.batch.s1[i]) % 128) return -1;
            unsigned set = 1u << (((uintptr_t)base % 128) / 16);
            for (int l = 0; l < p.ts.n; l++) {
                const uint64_t st = bytes(which == 0 ? p.ts.step_x[l] : p.ts.step_y[l]);
                if (st % 16) return -1;
                unsigned next = 0;
                for (int i = 0; i < p.ts.d[l] && i < 8; i++)
                    for (int r = 0; r < 8; r++)
                        if (set >> r & 1) next |= 1u << ((r + i * (st / 16)) % 8);
                set = next;
            }
            int w = 0;
            for (int r = 0; r < 8; r++)
                if (set >> r & 1) w = r;
            return w;
        };
        const int wx = p.a_kcontig ? worst(p.x, 0) : 0, wy = p.b_kcontig ? worst(p.y, 1) : 0;
        const int which = wx > 0 ? 1 : (wy > 0 ? 2 : 0);
        if (which) {
            const int64_t skip = (which == 1 ? wx : wy) * (16 / es);
            const int64_t stages = (p.K + skip + bk - 1) / bk;
            if (stages == stages0 || (stages == stages0 + 1 && stages0 >= 32)) {     // (an extra stage in 22 costs what whole lines gain)
                p.k_align = which;
                p.k_stages = (int32_t)stages;
            }
        }
    }
    if (f32) return tm == 128 ? dma::launch_layout<128, 128, 128, 2, 4, true>(p, stream) : dma::launch_layout<256, 256, 128, 2, 8, true>(p, stream);
    if (tm == 128) return dma::launch_layout<128, 128, 128, 2, 4, false>(p, stream);
    if (tn == 128) return dma::launch_layout<256, 128, 64, 3, 4, false>(p, stream);
    if (nw == 4) return dma::launch_layout<256, 256, 128, 2, 4, false>(p, stream);
    return dma::launch_layout<256, 256, 128, 2, 8, false>(p, stream);
}

// ------------------------------------------------------------------------------------------------
// Aggregation of tile-ordered partial slabs (AggTilesParams).
// The sums run over the slabs in ascending order in fp32 with one final cast, as in the dense-layout kernels
// (Section 4.2: the aggregation operator over the tuples that share an output block).
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ int64_t agg_tiles_offset(const DimList &g, int64_t idx, bool batch)
{
    int64_t o = 0;
    uint32_t rem = (uint32_t)idx;
    for (int i = g.n - 1; i >= 0; i--) {
        const uint32_t e = (uint32_t)g.ext[i], q = rem / e, k = rem - q * e;
        rem = q;
        o += (int64_t)k * (batch ? g.s2[i] : g.s1[i]);
    }
    return o;
}

// One workgroup per wave patch of an output tile, 32 rows at a time; the next 32 rows' slabs are fetched meanwhile.  (A workgroup
// per band of 32 rows across the whole tile, all loads issued at once, was 1.5 % faster on 16 slabs and 5-15 % slower on 2-8.)
template <int N>
__global__ __launch_bounds__(256) void k_aggregate_patches(const AggTilesParams p)
{
    __shared__ int64_t zr[128], zc[128];               // Z offsets of the patch's rows and columns
    __shared__ __attribute__((aligned(16))) float rows[32 * (128 + 4)];    // 32 rows of the patch on their way from register order to row order
    const int tid = threadIdx.x;
    const int WN = p.nw / 2, RT = p.tm / 64, NT = p.tn / WN / 32;
    const int PR = 32 * RT, PC = 32 * NT, pitch = PC + 4;
    // workgroup -> (output block, batch entry, tile row, tile column, wave of the join kernel)
    const uint32_t wave = blockIdx.x % (uint32_t)p.nw;
    int64_t T = blockIdx.x / (uint32_t)p.nw;
    const int64_t tile = T;
    const int64_t tile_n = T % p.tiles_n; T /= p.tiles_n;
    const int64_t tile_m = T % p.tiles_m; T /= p.tiles_m;
    const int64_t bidx = T % p.n_batch, grp = T / p.n_batch;
    const int64_t bz = group_offset_z(p.ts, grp) + agg_tiles_offset(p.batch, bidx, true);
    const int64_t row0 = tile_m * p.tm + (wave / WN) * PR, col0 = tile_n * p.tn + (wave % WN) * PC;
    if (tid < PR) zr[tid] = agg_tiles_offset(p.m, row0 + tid, false);
    else if (tid - PR < PC) zc[tid - PR] = agg_tiles_offset(p.n, col0 + (tid - PR), false);
    const float *src = p.partials + tile * ((int64_t)p.tm * p.tn) + (int64_t)wave * (RT * NT * 1024);
    const int lane = tid & 63, g4 = tid >> 6;          // chunk (k * 4 + g4) * 64 + lane of the patch, k = i * NT + j
    const int64_t slab4 = p.slab_stride / 4;
    const int orow = tid >> 3, oc0 = (tid & 7) * (PC / 8);    // on the way out: 8 threads per row, PC / 8 consecutive columns each
    // the sums of row tile i (NT chunks per thread); the loads of tile i + 1 are issued before tile i's rows are written out
    auto sums = [&](int i, f32x4 (&acc)[4]) {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (j >= NT) break;
            const f32x4 *s4 = (const f32x4 *)src + ((i * NT + j) * 4 + g4) * 64 + lane;
            if (N > 0) {
                f32x4 v[N > 0 ? N : 1];
#pragma unroll
                for (int a = 0; a < N; a++) v[a] = __builtin_nontemporal_load(s4 + a * slab4);
                acc[j] = v[0];
#pragma unroll
                for (int a = 1; a < N; a++) acc[j] += v[a];
            } else {
                acc[j] = __builtin_nontemporal_load(s4);
                for (int64_t a = 1; a < p.n_agg; a++) acc[j] += __builtin_nontemporal_load(s4 + a * slab4);
            }
        }
    };
    f32x4 cur[4], nxt[4];
    sums(0, cur);
    for (int i = 0; i < RT; i++) {
        __syncthreads();                               // the tables are there; the previous rows have been read
#pragma unroll
        for (int j = 0; j < 4; j++) {
            if (j >= NT) break;
            float *d = rows + (8 * g4 + 4 * (lane >> 5)) * pitch + j * 32 + (lane & 31);
            d[0] = cur[j].x; d[pitch] = cur[j].y; d[2 * pitch] = cur[j].z; d[3 * pitch] = cur[j].w;
        }
        if (i + 1 < RT) sums(i + 1, nxt);
        __syncthreads();
        const float *r = rows + orow * pitch + oc0;
        const int64_t zb = bz + zr[i * 32 + orow];
        if (p.vec) {                                    // Z runs along the columns: whole 16-byte pieces
            if (p.out_dtype == EG_BF16) {
                for (int c = 0; c < PC / 8; c += 8) {
                    const f32x4 a = *(const f32x4 *)(r + c), b = *(const f32x4 *)(r + c + 4);
                    uint4 o;
                    o.x = pack_bf16x2(a.x, a.y); o.y = pack_bf16x2(a.z, a.w); o.z = pack_bf16x2(b.x, b.y); o.w = pack_bf16x2(b.z, b.w);
                    *(uint4 *)((uint16_t *)p.out + zb + zc[oc0 + c]) = o;
                }
            } else {
                for (int c = 0; c < PC / 8; c += 4) *(f32x4 *)((float *)p.out + zb + zc[oc0 + c]) = *(const f32x4 *)(r + c);
            }
        } else {
            for (int c = 0; c < PC / 8; c++) store_elem(p.out, p.out_dtype, zb + zc[oc0 + c], r[c]);
        }
#pragma unroll
        for (int j = 0; j < 4; j++) cur[j] = nxt[j];
    }
}

int launch_aggregate_tiles(AggTilesParams &p, void *stream)
{
    if (!p.partials || !p.out) return fail(EG_ERR_NULL, "aggregation of tiles: NULL operand");
    const bool shape = (p.tm == 256 && p.tn == 256 && (p.nw == 8 || p.nw == 4)) || (p.tm == 256 && p.tn == 128 && p.nw == 4) || (p.tm == 128 && p.tn == 128 && p.nw == 4);
    if (!shape) return fail(EG_ERR_LIMIT, "aggregation of tiles: no join kernel writes %d x %d tiles with %d waves", p.tm, p.tn, p.nw);
    if (p.n_agg < 1 || p.tiles < 1 || p.tiles_m < 1 || p.tiles_n < 1 || p.n_batch < 1) return fail(EG_ERR_LIMIT, "aggregation of tiles: empty input");
    if (p.tiles % ((int64_t)p.tiles_m * p.tiles_n * p.n_batch)) return fail(EG_ERR_LIMIT, "aggregation of tiles: the tile count is no whole number of output blocks");
    if (p.slab_stride < p.tiles * p.tm * p.tn || p.slab_stride % 4 || ((uintptr_t)p.partials & 15)) return fail(EG_ERR_LIMIT, "aggregation of tiles: slabs overlap or are not 16-byte aligned");
    if (p.out_dtype != EG_F32 && p.out_dtype != EG_BF16) return fail(EG_ERR_DTYPE, "aggregation of tiles: result dtype");
    const int64_t wgs = p.tiles * p.nw;
    if (wgs >= (1ll << 31)) return fail(EG_ERR_LIMIT, "aggregation of tiles: %lld workgroups", (long long)wgs);
    // 16-byte stores along the rows: Z contiguous along the innermost column label in runs of whole pieces, everything else 8-aligned
    bool vec = p.n.s1[p.n.n - 1] == 1 && p.n.ext[p.n.n - 1] % 8 == 0 && ((uintptr_t)p.out & 15) == 0;
    for (int i = 0; i < p.m.n; i++) vec = vec && p.m.s1[i] % 8 == 0;
    for (int i = 0; i + 1 < p.n.n; i++) vec = vec && p.n.s1[i] % 8 == 0;
    for (int i = 0; i < p.batch.n; i++) vec = vec && p.batch.s2[i] % 8 == 0;
    for (int l = 0; l < p.ts.n; l++) vec = vec && p.ts.step_z[l] % 8 == 0;
    p.vec = vec ? 1 : 0;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)wgs), block(256);
    switch (p.n_agg) {
    case 2: EG_LAUNCH(k_aggregate_patches<2>, grid, block, 0, st, p); break;
    case 4: EG_LAUNCH(k_aggregate_patches<4>, grid, block, 0, st, p); break;
    case 8: EG_LAUNCH(k_aggregate_patches<8>, grid, block, 0, st, p); break;
    case 16: EG_LAUNCH(k_aggregate_patches<16>, grid, block, 0, st, p); break;
    default: EG_LAUNCH(k_aggregate_patches<0>, grid, block, 0, st, p); break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "k_aggregate_tiles launch failed: %s", hipGetErrorString(e));
    return EG_OK;
}

}  // namespace eg
