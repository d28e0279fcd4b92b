// Internal declarations shared by the host planner, the executor and the kernel launchers.
// Nothing in here is part of the public ABI (see include/eindecomp.h).
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "eindecomp.h"

namespace eg {

// ------------------------------------------------------------------------------------------------
// error reporting
// ------------------------------------------------------------------------------------------------
int fail(int code, const char *fmt, ...);   // records a thread-local message, returns code

// ------------------------------------------------------------------------------------------------
// device-visible parameter blocks (plain data, passed to kernels by value)
// ------------------------------------------------------------------------------------------------
constexpr int kMaxLabels = EG_MAX_LABELS;
constexpr int kMaxGroup = 4;     // labels per role group (batch / M / N / K) in the contraction kernel
constexpr int kMaxDims = 8;      // collapsed dimensions in the map / reduce kernels

// The join's tuple space (Section 4.3 of the paper): tuple t is the key over the schema in row-major
// order of I(d).  step_* = block extent * element stride of the label in X / Y / Z (0 when absent), so a
// block's base offset is sum_l key[l] * step[l].  agg_w[l] is the weight of key[l] in aggIdx, grp_w[l] its weight in
// the row-major index of the output block over the labels that are not aggregated.
struct TupleSpace {
    int32_t n;
    int32_t d[kMaxLabels];
    int32_t agg_w[kMaxLabels];
    int32_t grp_w[kMaxLabels];    // weight of key[l] in the index of the tuple's output block (0 for aggregated labels)
    int64_t step_x[kMaxLabels];
    int64_t step_y[kMaxLabels];
    int64_t step_z[kMaxLabels];
};

// Output addressing: when a vertex has a partitioned aggregated label the join kernel writes fp32
// partial blocks into slab aggIdx of the workspace ([n_agg][dense Z]); otherwise it writes the final
// tensor in its own dtype and strides.
struct OutSpec {
    void *ptr;            // device: slab 0 (partials) or the destination tensor
    int64_t slab_elems;   // element stride between slabs (partials only; 0 otherwise); at least the dense size of Z
    int32_t dtype;        // eg_dtype of what is stored through ptr
};

struct DimList {          // one role group of the contraction: block-level extents and strides
    int32_t n;
    int32_t ext[kMaxGroup];
    int64_t s0[kMaxGroup];   // batch: X, M: X, N: Y, K: X
    int64_t s1[kMaxGroup];   // batch: Y, M: Z, N: Z, K: Y
    int64_t s2[kMaxGroup];   // batch: Z
};

struct ContractParams {
    TupleSpace ts;
    DimList batch, m, n, k;
    int64_t M, N, K, n_batch;     // group sizes (products of block extents)
    int32_t a_kcontig;            // 1: X is contiguous along the innermost K label, 0: along innermost M label
    int32_t b_kcontig;            // 1: Y is contiguous along the innermost K label, 0: along innermost N label
    int32_t in_dtype;             // dtype of X and Y
    int32_t otimes, oplus;        // the vertex's scalar function and reduction; anything but multiply / sum runs on the vector ALU
    float alpha;
    const void *x;
    const void *y;
    OutSpec out;
    int64_t n_tuples;
    int64_t span_x, span_y;       // largest element offset inside one block of X / Y
    int32_t tiles_m, tiles_n;     // filled by the launcher
    int32_t out_vec;              // filled by the launcher: 1 = Z rows can be written as 16-byte vectors along N
    int32_t total_tiles, grid;    // filled by the launcher: output tiles over all tuples and batch entries; workgroups that share them
    int32_t force_kernel;         // 0: the launcher chooses; 1: register-staged kernel; 2: direct-to-LDS kernel wherever the layout allows (tr_set_contract_variant)
    int32_t force_tile_m, force_tile_n;   // 0: the launcher chooses; 128 x 128, 256 x 128 or 256 x 256: tile of the direct-to-LDS kernel
    int32_t force_waves;          // 0: the launcher chooses; 4 / 8: waves per workgroup of the 256 x 256 direct-to-LDS kernel
    int32_t tile_order;           // 1: partial slabs are written tile after tile in the accumulators' order (see AggTilesParams)
    int32_t k_stages;             // filled by the launcher of the direct-to-LDS kernel: stages per output tile
    int32_t k_align;              // filled by that launcher: 0: a tile's stages start at its block's first k; 1 / 2: on the 128-byte line of X / Y below it
};

// Aggregation of partial slabs that the direct-to-LDS contraction kernel wrote in tile order: a slab then holds the
// output tiles one after the other (output block, batch entry, tile row, tile column), each tile as the waves'
// accumulators lie in registers: 16-byte chunk (((wave * RT + i) * NT + j) * 4 + g) * 64 + lane holds rows
// 32 i + 8 g + 4 (lane / 32) .. + 3 and column 32 j + lane % 32 of the wave's patch, so the join kernel stores whole
// registers, 1 KiB per instruction, without a round trip through LDS, and the layout is undone here, where the
// kernel waits for memory anyway.  Same sums in the same order as the dense layout.
struct AggTilesParams {
    TupleSpace ts;                // step_z: the destination's
    DimList batch, m, n;          // batch.s2, m.s1, n.s1: the destination's element strides
    int64_t n_batch;
    int32_t tm, tn, nw;           // tile and waves of the join kernel
    int32_t tiles_m, tiles_n;
    int64_t tiles;                // per slab
    const float *partials;
    int64_t n_agg, slab_stride;   // slabs and the element stride between them
    void *out;
    int32_t out_dtype;
    int32_t vec;                  // filled by the launcher: the destination takes 16-byte stores along its rows
};

struct StridedDims {              // collapsed index space with per-operand element strides
    int32_t n;
    int32_t ext[kMaxDims];
    int64_t sx[kMaxDims], sy[kMaxDims], sz[kMaxDims];
};

struct MapParams {                // Z[z] = otimes(X[..], Y[..]) over one block per tuple
    TupleSpace ts;
    StridedDims dims;             // Z's block index space, outermost first; last dim is the vector dim
    int32_t binary, otimes;
    float alpha;
    int32_t dtx, dty;
    int32_t vec;                  // elements per lane along the last dim (1 = scalar path)
    const void *x;
    const void *y;
    OutSpec out;
    int64_t n_tuples;
    int64_t vecs_per_block;       // prod(ext[0..n-2]) * ceil(ext[n-1] / vec)
    int32_t tr;                   // 0: none.  1 / 2: X / Y has its stride-1 dimension at dims[td] instead of the last one
    int32_t td;                   //    (a transposed operand); it goes through LDS in 64 x 64 tiles, the other one is read along Z
};

struct ReduceParams {             // Z[z] = oplus over r of otimes(X[z, r], Y[z, r]); one wave-group per z
    TupleSpace ts;
    StridedDims zdims;            // output block index space (sz = destination strides)
    StridedDims rdims;            // reduced index space (sz unused); last dim contiguous in X when vec > 1
    int32_t binary, otimes, oplus;
    float alpha;
    int32_t dtx, dty;
    int32_t vec;
    const void *x;
    const void *y;
    OutSpec out;
    int64_t n_tuples;
    int64_t outs_per_block;
    int64_t red_elems;            // prod(rdims.ext)
    int32_t split;                // pieces per output's reduction range (1 = none); piece s lands in slab aggIdx*split+s
    int32_t col;                  // 1: the outputs' innermost dimension has stride 1 in X and Z; a lane holds 8 consecutive
                                  //    outputs and walks the reduced index space (rdims then has any strides)
};

struct GenericParams {            // any EinSum: one output element per lane, sequential loop over l_agg
    TupleSpace ts;
    StridedDims zdims;
    StridedDims rdims;
    int32_t binary, otimes, oplus;
    float alpha;
    int32_t dtx, dty;
    const void *x;
    const void *y;
    OutSpec out;
    int64_t n_tuples;
    int64_t outs_per_block;
    int64_t red_elems;
};

// A softmax over the last label, optionally preceded by alpha * x + y, computed row by row in one pass
// (the vertices max, exp(x - max), sum and division of Section 3's softmax, fused where the partitioning allows).
// An element-wise vertex behind a softmax chain that the chain's pass evaluates on the spot (D = L - max, log of the row sum,
// log-probabilities, the gradient P - Y, ...).  Operands are slots: 0 the chain's source value (after alpha * x + y, as its
// vertex stores it), 1 the row maximum, 2 the exponential, 3 the row sum, 4 the quotient, 5 / 6 a tensor of the result's
// shape read from memory, 8 + k the value of tail k (an earlier one).  Slots 1, 3 and row tails hold one value per row.
constexpr int kSoftmaxTails = 4, kSoftmaxExt = 2, kSoftmaxMore = kSoftmaxTails + kSoftmaxExt;
struct SoftmaxTail {
    int32_t op;                   // the vertex's scalar function
    float alpha;
    int32_t a, b;                 // operand slots (b = -1: one operand)
    int32_t row;                  // 1: one value per row (all operands are per-row slots)
    int32_t dt;                   // the vertex's dtype: values are rounded to it before anything uses them
    int32_t emit;                 // 1: the tensor is written (somebody outside the pass reads it, or it is an output)
    void *out;
};

struct SoftmaxParams {
    TupleSpace ts;                // steps of the source (x), of the added operand (y) and of the result (z)
    TupleSpace ts2;               // steps of the row maxima (x) and of the row sums (y) when those are written
    StridedDims rows;             // one entry per row label (extent > 1): sx source, sy added operand, sz result
    StridedDims stats;            // the same entries: sx row maxima, sy row sums
    int32_t n;                    // row length
    int64_t sx_last, sy_last, sz_last;   // element strides of the last label in source, added operand, result
    int32_t has_add, emit_max, emit_sum;
    int32_t dt_src, dt_add, dt_t, dt_e, dt_p, dt_max, dt_sum;   // storage dtypes; dt_t / dt_e: where the unfused vertices would round
    float alpha;
    const void *src;
    const void *add;
    void *p;
    void *row_max;
    void *row_sum;
    int64_t n_tuples, rows_per_block;
    int32_t vec;                  // filled by the launcher: 8 (16-byte accesses along the rows) or 1
    int32_t share_add;            // filled by the launcher: the rows of a workgroup take the same row of the added operand
    int32_t emit_p;               // 0: the quotient is not stored (only tails read it)
    // tails, and the addressing of the tensors they bring: entries 0 / 1 the tensors read (slots 5 / 6), 2 + k what tail k writes
    int32_t n_tail, n_ext;
    SoftmaxTail tail[kSoftmaxTails];
    const void *ext[kSoftmaxExt];
    int32_t dt_ext[kSoftmaxExt];
    int64_t more_last[kSoftmaxMore];                  // element stride along the last label
    int64_t more_rows[kSoftmaxMore][kMaxDims];        // ... along the entries of `rows`
    int64_t more_step[kSoftmaxMore][kMaxLabels];      // ... per block of the entries of `ts`
};

// Attention as one pass (see k_attention.hip): O[b.., q, :] = softmax_t(alpha * (alpha_qk * Q K^T) + mask) V per batch entry.
struct AttnParams {
    const void *q, *k, *v, *mask;
    void *o;
    uint8_t *cls;                     // with a mask: attention_mask_class_bytes(S, T) bytes of scratch, written and read by the launch
    int32_t cls_stride;               // filled by the launcher
    int32_t S, T, D;                  // query rows, key rows, head dimension
    int32_t nb0, nb1;                 // extents of up to two batch labels (nb1 varies fastest over blockIdx.y)
    int64_t q_sb0, q_sb1, q_ss;       // element strides of the batch labels and of the query label in Q (the head dimension has stride 1)
    int64_t k_sb0, k_sb1, k_st;       // ... of the key label in K
    int64_t v_sb0, v_sb1, v_st;
    int64_t o_sb0, o_sb1, o_ss;
    int64_t m_ss, m_st;               // element strides of the query and key labels in the mask (0: the mask lacks the label)
    int32_t has_mask, mask_dtype, mask_vec;   // mask_vec: filled by the launcher (16-byte reads of four consecutive keys)
    int32_t out_dtype;
    int32_t dt_t1, dt_t2;             // storage dtypes of the scores and of the scaled, masked scores: where the separate vertices round
    float alpha_qk, alpha;            // scalar of the first contraction, scalar of the scale-and-add vertex
};

struct AggregateParams {          // out[e] = oplus_a partials[a][e], ascending a, fp32, one final cast
    const float *partials;
    int64_t n_agg;
    int64_t slab_elems;           // elements of the output (and of every slab)
    int64_t slab_stride;          // element stride between slabs (>= slab_elems)
    int32_t oplus;
    int32_t out_dtype;
    void *out;
    int32_t contiguous;           // 1: out is dense row-major (vector path)
    StridedDims dims;             // out's index space (sz = out strides), used when not contiguous
};

// tr_execute runs every launcher twice: first with this thread-local flag set, so that each one makes all its checks
// and grid computations but enqueues nothing (an error then leaves device memory untouched), then for real.
bool validate_only();
void set_validate_only(bool on);
#define EG_LAUNCH(...) do { if (!eg::validate_only()) hipLaunchKernelGGL(__VA_ARGS__); } while (0)

// launchers (defined in the .hip files); each validates what its kernel assumes and returns eg_status
int launch_contract(ContractParams &p, void *stream);
int launch_contract_dma(ContractParams &p, void *stream);     // bf16, direct global->LDS staging; see k_contract_dma.hip
bool contract_dma_eligible(const ContractParams &p);
int launch_map(const MapParams &p, void *stream);
int launch_reduce_row(const ReduceParams &p, void *stream);
int launch_generic(const GenericParams &p, void *stream);
int launch_aggregate(const AggregateParams &p, void *stream);
int launch_softmax_rows(SoftmaxParams &p, void *stream);
int launch_attention(AttnParams &p, void *stream);
int launch_aggregate_tiles(AggTilesParams &p, void *stream);
bool contract_takes_dma(const ContractParams &p);                              // launch_contract will hand p to the direct-to-LDS kernel
void contract_dma_variant(const ContractParams &p, int &tm, int &tn, int &nw);   // ... which will run this tile shape and wave count
size_t attention_mask_class_bytes(int64_t S, int64_t T);

// ------------------------------------------------------------------------------------------------
// host-side graph
// ------------------------------------------------------------------------------------------------
struct Plan {                      // integer tables of one annotated vertex
    std::vector<int32_t> key, key_x, key_y, key_z, agg_idx, group;
    std::vector<int64_t> off_x, off_y, off_z;
    int64_t n_tuples = 0, n_agg = 1, n_groups = 1;
    bool valid = false;
};

struct Vertex {
    bool is_input = false;
    eg_dtype dtype = EG_F32;
    std::vector<int64_t> bound;            // b_Z (or the input's bound)
    // einsum vertices:
    std::string spec;
    std::vector<int> lx, ly, lz;           // schema index of every dimension of X / Y / Z
    std::vector<char> labels;              // schema: unique labels in first-appearance order
    std::vector<int64_t> lbound;           // bound per schema label
    std::vector<int32_t> d;                // partitioning per schema label
    std::vector<int> agg;                  // schema indices of aggregated labels (schema order)
    int otimes = EG_MUL, oplus = EG_AGG_SUM;
    double alpha = 1.0;
    int in[2] = {-1, -1};
    int n_in = 0;
    bool is_output = false;
    Plan plan;
};

}  // namespace eg

struct eg_graph {
    std::vector<eg::Vertex> v;
    std::vector<int> inputs;      // vertex ids of graph inputs, insertion order
    std::vector<int> outputs;     // marked outputs, marking order
    // executor state
    bool fuse = true;                               // fuse softmax chains where the partitioning allows (tr_set_fusion)
    bool fuse_attention = false;                    // scores, softmax chain and weighted sum as one pass (tr_set_fused_attention)
    bool tiled_partials = true;                     // partial slabs of whole-tile contractions in tile order (tr_set_tiled_partials)
    bool agg_in_kernel = false;                     // contractions sum over partitioned contracted labels inside the kernel (tr_set_fused_aggregation)
    int contract_kernel = 0, contract_tile_m = 0, contract_tile_n = 0, contract_waves = 0;   // tr_set_contract_variant (0: the launchers choose)
    bool profile = false;
    std::vector<void *> ev_start, ev_stop;          // hipEvent_t pool
    struct Launch { int vertex, stage, kernel; int64_t slabs; };   // slabs: partial slabs the launch wrote (join) or read (aggregation); 0 = none
    std::vector<Launch> launches;                   // of the last tr_execute
};

// defined in eg_exec.hip
void eg_release_events(eg_graph *g);
int eg_route_vertex(const eg_graph *g, int vertex);

struct eg_relation {
    void *ptr = nullptr;
    eg_dtype dtype = EG_F32;
    std::vector<int64_t> bound, stride;
    std::vector<int32_t> d;
};
