// Attention as one pass: the contraction Q x K^T, the softmax chain over the key label (optionally with the scale-and-add of a
// mask in front) and the contraction P x V of Section 3's attention, without the scores tensor ever leaving the chip.
//
// An alternative to the per-vertex path (off unless tr_set_fused_attention asks for it): the same EinSums, evaluated in
// another association.  Per batch entry (b, h) and block of 128 query rows a workgroup of four waves walks over the key
// rows in blocks of 64:
//   * scores: S^T = K Q^T on the matrix pipes (the matrix instruction gets K's fragment as its row operand), so a lane
//     holds ONE query (lane % 32) and, per 32 x 32 tile, sixteen keys; the two lanes l and l + 32 share a query;
//   * softmax statistics are then per-lane scalars: running maximum m and running sum l of the exponentials, rescaled
//     when a block raises the maximum (the usual streaming form of softmax; the row's final maximum and sum are those of
//     the max / sum vertices of the chain);
//   * the exponentials, rounded to bf16 as the chain's exp vertex stores them, are already laid out as the column operand
//     of the second product O^T = V^T P^T: which key a k-slot of the matrix instruction stands for is free as long as
//     both operands agree, and V's fragment is fetched from LDS with transposing reads whose row addresses follow the
//     layout the scores came out in;
//   * the scores are rounded where the separate vertices round them (after the product and after alpha * x + mask), the
//     division by the row sum happens once, at the end, on the fp32 accumulators (the separate vertices divide before the
//     second product and round P to bf16: results agree to a few bf16 units in the last place).
// K and V blocks go global memory -> registers -> LDS (swizzled for conflict-free fragment reads), the next block's loads
// issued before the current block's arithmetic.
// Requirements (checked by the launcher): bf16 Q, K, V with the head dimension contiguous and 32, 64 or 128 long, all
// other strides multiples of 8 elements, 16-byte aligned bases; the mask fp32 or bf16 with element strides per query and key.
#include <hip/hip_runtime.h>

#include "eg_device.h"

namespace eg {

typedef float at_f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 at_bf16x8 __attribute__((ext_vector_type(8)));
typedef short at_short4 __attribute__((ext_vector_type(4)));
typedef uint32_t at_u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 at_bf16x2 __attribute__((ext_vector_type(2)));
typedef float at_f32x4 __attribute__((ext_vector_type(4)));

#define EG_AT_LDS(p) ((__attribute__((address_space(3))) void *)(p))
constexpr float kAttnSlack = 5.f;                   // how far a row's maximum may rise above the value its exponentials are taken against
constexpr int kAttnMaxKeyBlocks = 1024;             // key blocks (of 64) whose mask classes a workgroup keeps in LDS

namespace {

__device__ __forceinline__ at_f32x16 at_mfma(const at_u32x4 &a, const at_u32x4 &b, at_f32x16 acc)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(at_bf16x8, a), __builtin_bit_cast(at_bf16x8, b), acc, 0, 0, 0);
}

// value of the partner lane (l ^ 32)
__device__ __forceinline__ float other_half(float v)
{
    const uint32_t u = __float_as_uint(v);
    const auto s = __builtin_amdgcn_permlane32_swap(u, u, false, false);    // lanes 32..63 of the first <-> lanes 0..31 of the second
    return __uint_as_float(threadIdx.x & 32 ? s[0] : s[1]);    // upper half: what arrived in the first; lower half: what arrived in the second
}

}  // namespace

// Class of a tile of the mask, 32 queries x 64 keys: what the pass may leave out there.
enum { AT_DEAD = 0,      // -inf throughout: the keys add nothing to these queries' maxima, sums or results
       AT_PLAIN = 1,     // zero throughout: nothing to load or add
       AT_MIXED = 2 };

// One workgroup per tile, eight rows per wave; lane = key, so a row's 64 entries are read as one contiguous piece when
// the key stride is 1.  cls[key block][query group], a byte per tile; groups beyond the last query (the row is padded to
// a multiple of four groups) come out dead.
__global__ __launch_bounds__(256) void k_attention_mask_classes(const AttnParams p)
{
    __shared__ int seen[4];
    const int group = blockIdx.x, blk = blockIdx.y, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int t = blk * 64 + lane;
    bool dead = true, zero = true;
#pragma unroll
    for (int r = 0; r < 8; r++) {
        const int row = group * 32 + wave * 8 + r;
        if (t < p.T && row < p.S) {
            const float m = load_elem(p.mask, p.mask_dtype, (int64_t)row * p.m_ss + (int64_t)t * p.m_st);
            dead = dead && m == -INFINITY;
            zero = zero && m == 0.f;
        }
    }
    const int mine = (__builtin_amdgcn_ballot_w64(!dead) != 0 ? 1 : 0) | (__builtin_amdgcn_ballot_w64(!zero) != 0 ? 2 : 0);
    if (lane == 0) seen[wave] = mine;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int all = seen[0] | seen[1] | seen[2] | seen[3];      // bit 0: some entry above -inf; bit 1: some entry not zero
        p.cls[(int64_t)blk * p.cls_stride + group] = !(all & 1) ? AT_DEAD : !(all & 2) ? AT_PLAIN : AT_MIXED;
    }
}

// One direct load from memory to LDS: the wave's 64 lanes fetch 16 bytes each from base + voff (zeros where voff + 16 goes
// beyond `bytes`) into the 1 KiB of LDS at lds_addr, lane after lane.  Written out by hand so that the compiler does not
// hold later LDS reads of the other stage until the load has landed; whoever reads the destination waits for vmcnt(0)
// and a barrier first.  M0 (the LDS base of a direct load) is put back.
__device__ __forceinline__ void at_load_lds(const void *base, uint32_t bytes, uint32_t lds_addr, uint32_t voff)
{
    const uint64_t b = (uint64_t)base;
    at_u32x4 rs;
    rs.x = __builtin_amdgcn_readfirstlane((uint32_t)b);
    rs.y = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) & 0xffffu;      // stride 0: a raw buffer
    rs.z = __builtin_amdgcn_readfirstlane(bytes);
    rs.w = 0x00020000u;
    const uint32_t l = __builtin_amdgcn_readfirstlane(lds_addr);
    uint32_t keep;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tbuffer_load_dwordx4 %2, %3, 0 offen lds\n\ts_mov_b32 m0, %0"
                 : "=&s"(keep) : "s"(l), "v"(voff), "s"(rs) : "memory");
}

// MASK: 0 = the group has no added operand; 1 = fp32 mask read 16 bytes (four consecutive keys) at a time; 2 = any
// mask, element by element.  RND: scores and scaled, masked scores are stored as bf16 by their vertices (else fp32).
template <int D, int MASK, bool RND>
__global__ __launch_bounds__(256, 2) void k_attention(const AttnParams p)
{
    constexpr int BM = 128, BN = 64;                   // query rows per workgroup, key rows per block
    constexpr int RB = D * 2, CH = D / 8;              // bytes and 16-byte chunks of a K / V row
    constexpr int RPB = RB >= 256 ? 1 : 256 / RB;      // rows per 256 bytes
    constexpr int TILE = BN * RB;                      // bytes of a K or V tile
    constexpr int NLD = TILE / 1024 / 4;               // direct loads (1 KiB each) per wave and tile
    constexpr int KT = D / 16, DT = D / 32;            // k-steps of the first product, 32-row tiles of O^T
    static_assert(D == 32 || D == 64 || D == 128, "head dimension");
    __shared__ __attribute__((aligned(1024))) char lds[2][2][TILE];     // two stages of a K tile and a V tile
    __shared__ uint8_t ctab[MASK ? kAttnMaxKeyBlocks : 4];              // per key block: the classes of the four query groups, two bits each
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lrow = lane & 31, lhalf = lane >> 5;
    // Workgroups go to the chip's eight dies in turn (each with an L2 of its own).  A batch entry's query blocks all run on
    // one die, so that its K and V are fetched from memory once; there they start with the last query block, which under a
    // causal mask has the most live key blocks.
    const int nq = (p.S + BM - 1) / BM, nbatch = p.nb0 * p.nb1;
    const int die = blockIdx.x & 7, turn = blockIdx.x >> 3;
    const int per_die = (nbatch + 7) / 8;
    const int bh = (turn % per_die) * 8 + die;
    if (bh >= nbatch) return;                          // the grid is rounded up to whole rounds over the dies
    const int qblk = nq - 1 - turn / per_die;
    const int b0 = bh / p.nb1, b1 = bh - b0 * p.nb1;
    const uint16_t *Q = (const uint16_t *)p.q + b0 * p.q_sb0 + b1 * p.q_sb1;
    const uint16_t *K = (const uint16_t *)p.k + b0 * p.k_sb0 + b1 * p.k_sb1;
    const uint16_t *V = (const uint16_t *)p.v + b0 * p.v_sb0 + b1 * p.v_sb1;
    const int qrow = qblk * BM + wave * 32 + lrow;                     // this lane's query
    const int qr = qrow < p.S ? qrow : p.S - 1;
    const int nblocks = (p.T + BN - 1) / BN;

    // K rows are read 16 bytes at a time by 16 lanes holding 16 consecutive rows: the chunk index is XOR-ed with the row
    // (per 256 bytes) so that they fall into 16 different bank groups.  V rows are read by the transposing 8-byte reads,
    // 4 consecutive rows x 32 bytes per 16 lanes: rows of a group of four are moved apart by multiples of 64 bytes.
    // A direct load fills LDS lane after lane, so the swizzle is applied to what a lane fetches: the lane whose 16 bytes
    // land in chunk position c of row r fetches chunk c ^ key(r) of that row.
#define EG_AT_KKEY(row) (((row) / RPB) % CH)
#define EG_AT_VKEY(row) ((((row) & 3) * (RB / 64)) & (CH - 1))
    uint32_t koff[NLD], voff[NLD];                     // byte offsets of this lane's fetches from the block's first row
#pragma unroll
    for (int c = 0; c < NLD; c++) {
        const int byte = (c * 4 + wave) * 1024 + lane * 16, row = byte / RB, ch = (byte % RB) >> 4;
        koff[c] = (uint32_t)(row * (int)p.k_st * 2 + ((ch ^ EG_AT_KKEY(row)) << 4));
        voff[c] = (uint32_t)(row * (int)p.v_st * 2 + ((ch ^ EG_AT_VKEY(row)) << 4));
    }
    // key block B -> LDS stage S: rows past the last key come in as zeros
#define EG_AT_ISSUE(B, S)                                                                                       \
    {                                                                                                           \
        const int left = p.T - (B) * BN < BN ? p.T - (B) * BN : BN;                                              \
        const uint32_t kbytes = (uint32_t)((left - 1) * (int)p.k_st * 2 + RB), vbytes = (uint32_t)((left - 1) * (int)p.v_st * 2 + RB); \
        const uint16_t *kb = K + (int64_t)(B) * BN * p.k_st, *vb = V + (int64_t)(B) * BN * p.v_st;                \
        _Pragma("unroll") for (int c = 0; c < NLD; c++) {                                                        \
            at_load_lds(kb, kbytes, (uint32_t)(uintptr_t)EG_AT_LDS(lds[S][0] + (c * 4 + wave) * 1024), koff[c]); \
            at_load_lds(vb, vbytes, (uint32_t)(uintptr_t)EG_AT_LDS(lds[S][1] + (c * 4 + wave) * 1024), voff[c]); \
        }                                                                                                       \
    }
#define EG_AT_LANDED() { __builtin_amdgcn_s_waitcnt(0x0f70); __syncthreads(); }   /* vmcnt(0): this wave's direct loads; then everybody's */

    // Q's fragments for all k-steps: column operand, lane = query, 8 consecutive d
    at_u32x4 qf[KT];
#pragma unroll
    for (int kk = 0; kk < KT; kk++) qf[kk] = *(const at_u32x4 *)(Q + (int64_t)qr * p.q_ss + 16 * kk + 8 * lhalf);
    // Waited for here, once: the compiler would otherwise wait for them in front of every block's first product, and
    // that wait (the counter runs in order) would take the direct loads of the next block with it.
    __builtin_amdgcn_s_waitcnt(0x0f70);

    at_f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; dt++)
#pragma unroll
        for (int r = 0; r < 16; r++) oacc[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    // classes of this workgroup's four query groups in every key block (a word per block in memory), two bits each
    if (MASK) {
        for (int b = tid; b < nblocks; b += 256) {
            const uint32_t w = *(const uint32_t *)(p.cls + (int64_t)b * p.cls_stride + qblk * 4);
            ctab[b] = (uint8_t)((w & 3) | ((w >> 6) & 0xc) | ((w >> 12) & 0x30) | ((w >> 18) & 0xc0));
        }
        __syncthreads();
    }
#define EG_AT_SKIP_DEAD(B) { if (MASK) while ((B) < nblocks && ctab[B] == 0) (B)++; }
    // Key blocks that are dead for all four query groups are left out altogether.  A live block's tiles are in LDS stage
    // `stage` while the block is worked on; the next live block's travel from memory into the other stage meanwhile, which
    // the barrier at the end of the previous block has freed of its readers.
    int blk = 0, stage = 0;
    EG_AT_SKIP_DEAD(blk)
    int nxt = blk + 1;
    if (blk < nblocks) {
        EG_AT_ISSUE(blk, 0)
        EG_AT_SKIP_DEAD(nxt)
        EG_AT_LANDED()
    }
    while (blk < nblocks) {
        if (nxt < nblocks) { EG_AT_ISSUE(nxt, stage ^ 1) }
        const int my = MASK ? __builtin_amdgcn_readfirstlane((ctab[blk] >> (2 * wave)) & 3) : (int)AT_PLAIN;
        const bool tail = blk == nblocks - 1 && (p.T & (BN - 1)) != 0;
        const char *ks = lds[stage][0], *vs = lds[stage][1];
        if (my != AT_DEAD) {
            // ---- the mask's entries of a mixed tile, fetched first so that they travel under the scores' product ----
            float mk[2][16];
            const int64_t mrow = (int64_t)qr * p.m_ss;
            if (MASK == 1 && my == AT_MIXED) {
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int g = 0; g < 4; g++) {
                        int t0 = blk * BN + i * 32 + 8 * g + 4 * lhalf;
                        t0 = t0 < p.T ? t0 : p.T - 4;       // T is a multiple of four here; keys past the end are set to -inf below
                        const at_f32x4 f = *(const at_f32x4 *)((const float *)p.mask + mrow + t0);
                        mk[i][4 * g] = f[0]; mk[i][4 * g + 1] = f[1]; mk[i][4 * g + 2] = f[2]; mk[i][4 * g + 3] = f[3];
                    }
            }

            // ---- scores: S^T (keys x queries) = K Q^T; the fragments of the next k-step are read under this one's products ----
            at_f32x16 sacc[2];
            const at_f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            at_u32x4 kf[KT][2];
#define EG_AT_KFRAG(KK, I) (*(const at_u32x4 *)(ks + ((I) * 32 + lrow) * RB + (((2 * (KK) + lhalf) ^ EG_AT_KKEY((I) * 32 + lrow)) << 4)))
#pragma unroll
            for (int kk = 0; kk < KT; kk++) {
                kf[kk][0] = EG_AT_KFRAG(kk, 0);
                kf[kk][1] = EG_AT_KFRAG(kk, 1);
            }
            __builtin_amdgcn_sched_barrier(0);          // all reads on their way before the first product waits for one
#pragma unroll
            for (int kk = 0; kk < KT; kk++) {
                sacc[0] = at_mfma(kf[kk][0], qf[kk], kk == 0 ? zero : sacc[0]);
                sacc[1] = at_mfma(kf[kk][1], qf[kk], kk == 0 ? zero : sacc[1]);
            }
#undef EG_AT_KFRAG

            // ---- the chain's element-wise steps on this lane's 32 keys: key of (i, r) = 32 i + 8 (r / 4) + 4 half + r % 4 ----
            float x[2][16];
#pragma unroll
            for (int i = 0; i < 2; i++) {
#pragma unroll
                for (int r = 0; r < 16; r++) x[i][r] = sacc[i][r];
                if (p.alpha_qk != 1.f)
#pragma unroll
                    for (int r = 0; r < 16; r++) x[i][r] *= p.alpha_qk;
                if (RND)
#pragma unroll
                    for (int r = 0; r < 16; r += 2) round_pair_bf16(x[i][r], x[i][r + 1]);
            }
            if (MASK) {
                if (my == AT_MIXED) {
                    if (MASK == 2) {
#pragma unroll
                        for (int i = 0; i < 2; i++)
#pragma unroll
                            for (int r = 0; r < 16; r++) {
                                int t = blk * BN + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
                                t = t < p.T ? t : p.T - 1;
                                mk[i][r] = load_elem(p.mask, p.mask_dtype, mrow + (int64_t)t * p.m_st);
                            }
                    }
#pragma unroll
                    for (int i = 0; i < 2; i++)
#pragma unroll
                        for (int r = 0; r < 16; r++) x[i][r] = p.alpha * x[i][r] + mk[i][r];
                } else {
#pragma unroll
                    for (int i = 0; i < 2; i++)
#pragma unroll
                        for (int r = 0; r < 16; r++) x[i][r] = p.alpha * x[i][r];
                }
                if (RND)
#pragma unroll
                    for (int i = 0; i < 2; i++)
#pragma unroll
                        for (int r = 0; r < 16; r += 2) round_pair_bf16(x[i][r], x[i][r + 1]);
            }
            if (tail) {                                 // keys past the end take no part
                asm volatile("" ::: "memory");          // a branch taken once, not 32 selects in every block
#pragma unroll
                for (int i = 0; i < 2; i++)
#pragma unroll
                    for (int r = 0; r < 16; r++)
                        if (blk * BN + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3) >= p.T) x[i][r] = -INFINITY;
            }
            float bmax = -INFINITY;
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int r = 0; r < 16; r++) bmax = fmaxf(bmax, x[i][r]);
            bmax = fmaxf(bmax, other_half(bmax));
            // The reference value follows the maximum only when that has risen by more than kAttnSlack since it was last set:
            // exponentials then reach e^slack at most, and the accumulators are rescaled on few blocks instead of nearly all.
            const float m_new = bmax - m_run > kAttnSlack ? bmax : m_run;           // (-inf - -inf is NaN: stays at -inf)
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;                  // a row that has seen only -inf so far
            const float scale = __builtin_amdgcn_exp2f((m_run - m_safe) * kLog2e);  // 0 while m_run is -inf
            const float nml = -(m_safe * kLog2e);
            float psum = 0.f;
            at_u32x4 pf[2][2];                          // exponentials as bf16: column operand of the second product
            const at_bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        const float a = exp_sub_scaled(x[i][8 * j + 2 * e], nml), b = exp_sub_scaled(x[i][8 * j + 2 * e + 1], nml);
                        w[e] = pack_bf16x2(a, b);
                        psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(at_bf16x2, w[e]), ones, psum, false);   // the sum runs over the stored values
                    }
                    pf[i][j].x = w[0]; pf[i][j].y = w[1]; pf[i][j].z = w[2]; pf[i][j].w = w[3];
                }
            psum += other_half(psum);
            l_run = l_run * scale + psum;
            m_run = m_new;
            if (__builtin_amdgcn_ballot_w64(scale != 1.f) != 0) {      // some query's maximum rose
                asm volatile("" ::: "memory");          // (a branch: rare after the first blocks)
#pragma unroll
                for (int dt = 0; dt < DT; dt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) oacc[dt][r] *= scale;
            }

            // ---- O^T (head dimension x queries) += V^T P^T ---------------------------------------------
            // k-slot (half h, i) of step (i32, j) stands for key 32 i32 + 16 j + 8 (i / 4) + 4 h + i % 4, as the scores came out;
            // step n = (i32, j, dt), the fragment of step n + 1 read under step n's product
            const int s16 = lane & 15;
            typedef short at_short8 __attribute__((ext_vector_type(8)));
            auto vfrag = [&](int n) -> at_u32x4 {
                const int ij = n / DT, dt = n % DT, i = ij >> 1, j = ij & 1;
                const int col = dt * 32 + 16 * ((lane >> 4) & 1) + 4 * (s16 & 3);           // first of this lane's four d
                at_short4 part[2];
#pragma unroll
                for (int sec = 0; sec < 2; sec++) {
                    const int row = i * 32 + 16 * j + 8 * sec + 4 * lhalf + (s16 >> 2);
                    const char *addr = vs + row * RB + (((col >> 3) ^ EG_AT_VKEY(row)) << 4) + ((col & 7) << 1);
                    part[sec] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) at_short4 *)((__attribute__((address_space(3))) void *)addr));
                }
                const at_short8 both = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
                return __builtin_bit_cast(at_u32x4, both);
            };
            at_u32x4 vf[2];
            vf[0] = vfrag(0);
#pragma unroll
            for (int n = 0; n < 4 * DT; n++) {
                if (n + 1 < 4 * DT) vf[(n + 1) & 1] = vfrag(n + 1);
                const int ij = n / DT, dt = n % DT;
                oacc[dt] = at_mfma(vf[n & 1], pf[ij >> 1][ij & 1], oacc[dt]);
            }
        }
        blk = nxt;
        if (blk < nblocks) {
            nxt = blk + 1;
            EG_AT_SKIP_DEAD(nxt)
            EG_AT_LANDED()
            stage ^= 1;
        }
    }

    // ---- division by the row sum, store: lane holds query qrow and, per tile, d = 32 dt + 8 (r / 4) + 4 half + r % 4 ----
    const float inv = 1.f / l_run;                     // a row with no finite score: 0 x inf = NaN, as 0 / 0 in the chain's division
    const int64_t ob = b0 * p.o_sb0 + b1 * p.o_sb1 + (int64_t)qr * p.o_ss;
    const bool ok = qrow < p.S;
#pragma unroll
    for (int dt = 0; dt < DT; dt++) {
        if (p.out_dtype == EG_BF16) {
#pragma unroll
            for (int gp = 0; gp < 2; gp++) {
                const int r0 = 8 * gp;
                uint32_t x0 = pack_bf16x2(oacc[dt][r0] * inv, oacc[dt][r0 + 1] * inv), x1 = pack_bf16x2(oacc[dt][r0 + 2] * inv, oacc[dt][r0 + 3] * inv);
                uint32_t y0 = pack_bf16x2(oacc[dt][r0 + 4] * inv, oacc[dt][r0 + 5] * inv), y1 = pack_bf16x2(oacc[dt][r0 + 6] * inv, oacc[dt][r0 + 7] * inv);
                // the upper half-wave's first group against the lower half-wave's second: every lane ends up with 8 consecutive d
                const auto s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
                const auto s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
                uint4 o;
                o.x = s0[0]; o.y = s1[0]; o.z = s0[1]; o.w = s1[1];
                if (ok) *(uint4 *)((uint16_t *)p.o + ob + dt * 32 + 16 * gp + 8 * lhalf) = o;
            }
        } else {
#pragma unroll
            for (int g = 0; g < 4; g++) {
                float4 o = make_float4(oacc[dt][4 * g] * inv, oacc[dt][4 * g + 1] * inv, oacc[dt][4 * g + 2] * inv, oacc[dt][4 * g + 3] * inv);
                if (ok) *(float4 *)((float *)p.o + ob + dt * 32 + 8 * g + 4 * lhalf) = o;
            }
        }
    }
}

#undef EG_AT_ISSUE
#undef EG_AT_LANDED
#undef EG_AT_SKIP_DEAD
#undef EG_AT_KKEY
#undef EG_AT_VKEY

size_t attention_mask_class_bytes(int64_t S, int64_t T)
{
    const int64_t groups = ((S + 31) / 32 + 3) / 4 * 4, blocks = (T + 63) / 64;
    return (size_t)(groups * blocks);
}

template <int D>
static void launch_attention_d(const AttnParams &p, int mask, bool rnd, dim3 grid, hipStream_t st)
{
    if (mask == 0) { if (rnd) EG_LAUNCH((k_attention<D, 0, true>), grid, dim3(256), 0, st, p); else EG_LAUNCH((k_attention<D, 0, false>), grid, dim3(256), 0, st, p); }
    else if (mask == 1) { if (rnd) EG_LAUNCH((k_attention<D, 1, true>), grid, dim3(256), 0, st, p); else EG_LAUNCH((k_attention<D, 1, false>), grid, dim3(256), 0, st, p); }
    else { if (rnd) EG_LAUNCH((k_attention<D, 2, true>), grid, dim3(256), 0, st, p); else EG_LAUNCH((k_attention<D, 2, false>), grid, dim3(256), 0, st, p); }
}

int launch_attention(AttnParams &p, void *stream)
{
    if (!p.q || !p.k || !p.v || !p.o || (p.has_mask && (!p.mask || !p.cls))) return fail(EG_ERR_NULL, "attention kernel: NULL operand");
    if (p.S < 1 || p.T < 1 || p.nb0 < 1 || p.nb1 < 1) return fail(EG_ERR_LIMIT, "attention kernel: empty index space");
    if (p.D != 32 && p.D != 64 && p.D != 128) return fail(EG_ERR_LIMIT, "attention kernel: head dimension %d (32, 64 or 128)", p.D);
    const int64_t strides[] = {p.q_sb0, p.q_sb1, p.q_ss, p.k_sb0, p.k_sb1, p.k_st, p.v_sb0, p.v_sb1, p.v_st, p.o_sb0, p.o_sb1, p.o_ss};
    for (int64_t s : strides)
        if (s % 8 || s < 0) return fail(EG_ERR_LIMIT, "attention kernel: strides must be non-negative multiples of 8 elements");
    if (((uintptr_t)p.q & 15) || ((uintptr_t)p.k & 15) || ((uintptr_t)p.v & 15) || ((uintptr_t)p.o & 15))
        return fail(EG_ERR_LIMIT, "attention kernel: operands must be 16-byte aligned");
    if (p.has_mask && p.dt_t1 != p.dt_t2) return fail(EG_ERR_LIMIT, "attention kernel: the scores and the scaled, masked scores must have one storage dtype");
    const int64_t qblocks = ((int64_t)p.S + 127) / 128, nb = (int64_t)p.nb0 * p.nb1, kblocks = ((int64_t)p.T + 63) / 64;
    if (p.k_st >= (1ll << 23) || p.v_st >= (1ll << 23)) return fail(EG_ERR_LIMIT, "attention kernel: key strides of K and V must stay below 2^23 elements");
    if (p.has_mask && kblocks > kAttnMaxKeyBlocks) return fail(EG_ERR_LIMIT, "attention kernel: at most %d keys with an added operand", kAttnMaxKeyBlocks * 64);
    if (qblocks >= (1ll << 29) || nb >= (1ll << 31) || kblocks > 65535)
        return fail(EG_ERR_LIMIT, "attention kernel: %lld query blocks x %lld batch entries, %lld key blocks", (long long)qblocks, (long long)nb, (long long)kblocks);
    p.mask_vec = p.has_mask && p.m_st == 1 && p.mask_dtype == EG_F32 && ((uintptr_t)p.mask & 15) == 0 && p.m_ss % 4 == 0 && p.T % 4 == 0;
    hipStream_t st = (hipStream_t)stream;
    if (p.has_mask) {
        if ((uintptr_t)p.cls & 3) return fail(EG_ERR_LIMIT, "attention kernel: the class table must be 4-byte aligned");
        p.cls_stride = (int32_t)(qblocks * 4);
        EG_LAUNCH(k_attention_mask_classes, dim3((unsigned)(qblocks * 4), (unsigned)kblocks), dim3(256), 0, st, p);
    }
    const int64_t wgs = qblocks * ((nb + 7) / 8 * 8);
    if (wgs >= (1ll << 31)) return fail(EG_ERR_LIMIT, "attention kernel: %lld workgroups", (long long)wgs);
    const dim3 grid((unsigned)wgs);
    const int mask = !p.has_mask ? 0 : p.mask_vec ? 1 : 2;
    const bool rnd = p.dt_t1 == EG_BF16;
    if (p.D == 128) launch_attention_d<128>(p, mask, rnd, grid, st);
    else if (p.D == 64) launch_attention_d<64>(p, mask, rnd, grid, st);
    else launch_attention_d<32>(p, mask, rnd, grid, st);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(EG_ERR_HIP, "k_attention launch failed: %s", hipGetErrorString(e));
    return EG_OK;
}

}  // namespace eg
