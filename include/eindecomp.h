/*
 * eindecomp.h - C ABI of the MI355X tensor-relational einsum executor.
 *
 * The library runs an already-decomposed graph of extended Einstein-summation
 * vertices (arxiv 2410.02682) on one GPU.  Per vertex it follows the rewrite of
 * Section 4.3 of the paper: the inputs are tensor relations (Section 4.1: keyed
 * blocks fixed by a bound vector b and a partitioning vector d); a join matches
 * blocks whose keys agree on shared labels and runs the per-block kernel K on
 * every matched pair; an aggregation reduces, with the vertex's (+), the partial
 * blocks that belong to the same output key, in ascending order of the key over
 * the aggregated labels.
 *
 * Conventions
 *   - All functions return EG_OK (0) or a negative eg_status.  No exception
 *     crosses the ABI; eg_last_error() gives a thread-local message for the
 *     last failing call.
 *   - "host" / "device" is stated for every pointer.  Device buffers and the HIP
 *     stream always belong to the caller; the library never allocates, frees or
 *     synchronises device memory.  Handles (eg_graph, eg_relation) own host
 *     memory only and are released by their *_destroy call.
 *   - All validation happens on the host before any launch: tr_execute routes
 *     every vertex and runs every kernel launcher's checks (shapes, limits,
 *     grid sizes) once without launching before it enqueues anything, so a
 *     call that fails for such a reason leaves device memory untouched.  Only
 *     an error of the HIP runtime at an actual launch (EG_ERR_HIP) can occur
 *     after earlier vertices have been enqueued.
 *   - Tensors are dense with element strides (row-major unless strides are
 *     given).  A block of a relation is a strided view into that buffer, so
 *     partitioning and repartitioning move no data.
 *   - A partitioning vector is given per UNIQUE label of the vertex, in order of
 *     first appearance over l_X then l_Y (the schema of the natural join,
 *     Section 4.3): for "ij,jk->ik" the vector (2,2,2) is the paper's
 *     d = [2,2,2,2] with the co-partitioning constraint of Section 6 applied.
 *   - Tuple order (the paper leaves it open): row-major over I(d) on that
 *     schema, last label fastest.  aggIdx is the row-major rank of the key
 *     restricted to the aggregated labels; group is the rank of the key
 *     restricted to l_Z (in l_Z order) within I(d_Z).
 */
#ifndef EINDECOMP_H
#define EINDECOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EG_MAX_RANK 8      /* dimensions per tensor */
#define EG_MAX_LABELS 12   /* unique labels per vertex */

typedef enum {
    EG_OK = 0,
    EG_ERR_NULL = -1,            /* a required pointer is NULL */
    EG_ERR_BAD_SPEC = -2,        /* spec string malformed, operand count mismatch */
    EG_ERR_REPEATED_LABEL = -3,  /* a label occurs twice inside one operand (Section 3 excludes it) */
    EG_ERR_BROADCAST = -4,       /* an output label occurs in no input (Section 3 excludes it) */
    EG_ERR_BAD_BOUND = -5,       /* rank/bound mismatch, or a shared label with two different bounds */
    EG_ERR_BAD_PARTITION = -6,   /* wrong length, entry < 1 */
    EG_ERR_INDIVISIBLE = -7,     /* d[i] does not divide b[i] */
    EG_ERR_DTYPE = -8,           /* unsupported dtype or dtype mismatch with a bound relation */
    EG_ERR_WORKSPACE = -9,       /* workspace missing, misaligned or too small */
    EG_ERR_BAD_VERTEX = -10,     /* vertex id out of range / not an einsum vertex / wrong binding count */
    EG_ERR_BAD_OP = -11,         /* (x)/(+) combination not valid for this spec */
    EG_ERR_HIP = -12,            /* a HIP runtime call failed */
    EG_ERR_LIMIT = -13           /* exceeds EG_MAX_RANK / EG_MAX_LABELS / 32-bit tile grid limits */
} eg_status;

typedef enum { EG_F32 = 0, EG_BF16 = 1 } eg_dtype;

/* (+): the aggregation operator; must be associative and commutative (Section 3). */
typedef enum { EG_AGG_NONE = 0, EG_AGG_SUM = 1, EG_AGG_MAX = 2 } eg_agg;

/* (x): the scalar function applied to joined values (Section 3).  alpha is the one scalar
 * parameter a vertex carries.  Binary: */
typedef enum {
    EG_MUL = 0,        /* alpha * x * y      (with EG_AGG_SUM: a contraction)            */
    EG_ADD = 1,        /* alpha * x + y      (scale then add: scaled scores + mask)      */
    EG_SUB = 2,        /* alpha * (x - y)                                                */
    EG_DIV = 3,        /* x / y                                                          */
    EG_SQDIFF = 4,     /* (x - y)^2          (squared L2 distance, Section 3)            */
    EG_ABSDIFF = 5,    /* |x - y|            (L-infinity distance with EG_AGG_MAX)       */
    EG_EXP_SUB = 6,    /* exp(x - y)         (softmax numerator, Section 3)              */
    EG_RELU_GRAD = 7,  /* x if y > 0 else 0                                              */
    EG_SILU_MUL = 8,   /* x * sigmoid(x) * y                                             */
    /* unary maps: */
    EG_IDENT = 32,     /* x                                                              */
    EG_SCALE = 33,     /* alpha * x                                                      */
    EG_RELU = 34,      /* max(x, 0)                                                      */
    EG_EXP = 35,       /* exp(x)                                                         */
    EG_LOG = 36        /* log(x)                                                         */
} eg_join;

typedef struct eg_graph eg_graph;        /* an EinGraph annotated with partitioning vectors (Sections 5-6) */
typedef struct eg_relation eg_relation;  /* a tensor relation: b, d, dtype and a borrowed device pointer   */

/* Which device kernel family a vertex is routed to (reported by einsum_graph_plan). */
typedef enum {
    EG_KERNEL_NONE = 0,
    EG_KERNEL_CONTRACT_MFMA = 1,   /* (x)=mul, (+)=sum as a strided batched matrix product on MFMA   */
    EG_KERNEL_MAP = 2,             /* no aggregated label: elementwise map / binary join             */
    EG_KERNEL_REDUCE_ROW = 3,      /* aggregated labels are the contiguous tail of X: wave reductions */
    EG_KERNEL_GENERIC = 4,         /* any EinSum: one output element per lane, loop over l_agg       */
    EG_KERNEL_CONTRACT_ALU = 5,    /* contraction-shaped EinSum with another (x)/(+) pair (squared L2, L-infinity, ...): LDS tiles, vector ALU */
    EG_KERNEL_SOFTMAX_FUSED = 6,   /* the softmax vertices max, exp(x - max), sum, division (a preceding alpha*x + y, element-wise vertices behind it) in one pass per row */
    EG_KERNEL_ATTENTION_FUSED = 7, /* Section 3's attention, scores contraction to weighted sum, in one pass (tr_set_fused_attention) */
    EG_KERNEL_AGGREGATE_TILES = 8  /* reported for an aggregation launch that read tile-ordered partial slabs (tr_set_tiled_partials) */
} eg_kernel_kind;

/* Read-only view of one vertex's plan.  All pointers are host memory owned by the graph and stay
 * valid until the vertex's partition changes or the graph is destroyed. */
typedef struct {
    int32_t n_labels;                    /* unique labels (schema of the join) */
    char    labels[EG_MAX_LABELS];       /* their characters, schema order */
    int64_t bound[EG_MAX_LABELS];        /* b per unique label */
    int32_t d[EG_MAX_LABELS];            /* partitioning per unique label */
    int32_t rank_x, rank_y, rank_z;      /* rank_y = 0 for a unary vertex */
    int32_t d_x[EG_MAX_RANK], d_y[EG_MAX_RANK], d_z[EG_MAX_RANK];   /* d[l_X; l_XY] etc. (Section 4.3) */
    int64_t bound_z[EG_MAX_RANK];        /* b_Z = b_XY[l_Z; l_XY] */
    int64_t block_x[EG_MAX_RANK], block_y[EG_MAX_RANK], block_z[EG_MAX_RANK];  /* sub-tensor bounds b/d */
    int64_t n_tuples;                    /* N = prod d over the schema (Section 6) */
    int64_t n_agg;                       /* prod d over the aggregated labels (Section 7) */
    int64_t n_groups;                    /* N / n_agg = number of output blocks */
    int32_t kernel;                      /* eg_kernel_kind */
    int32_t repart_x, repart_y;          /* 1 if the producer's d_Z differs from this vertex's d_X / d_Y (Section 5) */
    /* per tuple, tuple-major, host: */
    const int32_t *key;                  /* [n_tuples][n_labels] key over the schema */
    const int32_t *key_x;                /* [n_tuples][rank_x] */
    const int32_t *key_y;                /* [n_tuples][rank_y] */
    const int32_t *key_z;                /* [n_tuples][rank_z] */
    const int32_t *agg_idx;              /* [n_tuples] */
    const int32_t *group;                /* [n_tuples] */
    const int64_t *off_x;                /* [n_tuples] element offset of the X block in a dense row-major X */
    const int64_t *off_y;                /* [n_tuples] likewise for Y (0 if unary) */
    const int64_t *off_z;                /* [n_tuples] likewise for the Z block in a dense row-major Z */
} eg_plan_view;

/* ---- EinGraph construction (Section 5: one triple (bound, EinSum, inputs) per vertex) ------------------- */

/* Creates an empty graph.  *g (host) receives the handle. */
int einsum_graph_create(eg_graph **g);

/* Adds a graph input (a vertex with empty EinSum and no inputs).  bound: host, `rank` entries, each >= 1.
 * *vertex receives its id.  Vertex ids count up from 0 in insertion order, which is a topological order. */
int einsum_graph_add_input(eg_graph *g, int rank, const int64_t *bound, eg_dtype dtype, int *vertex);

/* Adds an EinSum vertex.  spec (host, NUL-terminated): "ij,jk->ik" (binary) or "ij->i" (unary); one
 * character per label; "->" followed by nothing denotes a rank-0 output.  inputs (host): n_inputs (1 or 2)
 * ids of earlier vertices, ordered as in the spec (the EinSum need not be commutative).  The output bound
 * is deduced (b_Z = b_XY[l_Z; l_XY]).  oplus must be SUM or MAX when some input label is missing from the
 * output and is ignored otherwise.  The partitioning defaults to all ones. */
int einsum_graph_add_einsum(eg_graph *g, const char *spec, eg_join otimes, eg_agg oplus, double alpha,
                            const int *inputs, int n_inputs, eg_dtype out_dtype, int *vertex);

/* Annotates a vertex with its partitioning vector (Section 6), one entry per unique label in schema order.
 * d: host.  Rejects entries < 1 (EG_ERR_BAD_PARTITION) and entries that do not divide the label's bound
 * (EG_ERR_INDIVISIBLE; the paper only ever divides evenly). */
int einsum_graph_set_partition(eg_graph *g, int vertex, const int32_t *d, int n_unique_labels);

/* Marks a vertex as a graph output: tr_execute writes it into a caller-provided relation instead of the
 * workspace.  Outputs are bound in the order they were marked. */
int einsum_graph_mark_output(eg_graph *g, int vertex);

/* Fills *out (host, caller-owned struct) with the vertex's plan tables; see eg_plan_view. */
int einsum_graph_plan(eg_graph *g, int vertex, eg_plan_view *out);

/* Number of vertices, or a negative status. */
int einsum_graph_num_vertices(const eg_graph *g);

void einsum_graph_destroy(eg_graph *g);

/* ---- Tensor relations (Section 4.1) ---------------------------------------------------------------------- */

/* Views the dense tensor at dev_ptr (device, borrowed) as the tensor relation with bound `bound` and
 * partitioning `d` (host arrays, `rank` entries).  strides_or_null: element strides (host) or NULL for
 * row-major.  No data moves: block <k> is the strided view starting at sum_i k[i]*(b[i]/d[i])*stride[i]. */
int tensor_partition(void *dev_ptr, eg_dtype dtype, int rank, const int64_t *bound,
                     const int64_t *strides_or_null, const int32_t *d, eg_relation **rel);

/* Descriptor of block `key` (host, rank entries): element offset, block bound and strides (host outputs,
 * rank entries each; any may be NULL). */
int tensor_relation_block(const eg_relation *rel, const int32_t *key,
                          int64_t *offset, int64_t *bound, int64_t *strides);

/* Releases the handle; never touches the device buffer. */
void tensor_relation_destroy(eg_relation *rel);

/* ---- Execution (Sections 4.2-4.3, 5) ----------------------------------------------------------------------- */

/* Bytes of device workspace tr_execute needs for the graph as currently annotated: fp32 partial slabs
 * ([n_agg][dense Z] per vertex with a partitioned aggregated label) plus every intermediate vertex that
 * is not a marked output, with buffers reused once their last consumer has run.  Where a vertex has few
 * outputs under a long reduction, the execution cuts that reduction into further pieces of its own (more
 * partial slabs, added in ascending order like the others); their space is counted here. */
int tr_workspace_bytes(eg_graph *g, size_t *bytes);

/* Runs every vertex in topological order on `hip_stream` (a hipStream_t, may be NULL for the default
 * stream), asynchronously.  inputs: one relation per graph input in insertion order; outputs: one relation
 * per marked output in marking order (both host arrays of handles).  Bounds and dtypes must match the
 * graph's.  A relation whose d differs from what the consuming vertex needs is repartitioned (Section 5);
 * with strided-view blocks that is a change of tables only.  workspace: device, 256-byte aligned, at least
 * tr_workspace_bytes(). */
int tr_execute(eg_graph *g, eg_relation *const *inputs, int n_inputs,
               eg_relation *const *outputs, int n_outputs,
               void *workspace, size_t workspace_bytes, void *hip_stream);

/* tr_execute for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same graph, same relations, same kernels and results as
 * tr_execute; the partial slabs and intermediates live in a workspace that belongs to the library: a file-scope
 * device array of tr_static_workspace_bytes() = 32 MiB, of which every GPU the library runs on holds its own copy
 * until the process ends.  The call allocates nothing on the device and calls no allocating routine; the array's
 * address on the current device is looked up at the first call on that device.  A graph that needs more
 * (tr_workspace_bytes) is rejected with EG_ERR_WORKSPACE before anything is launched: use tr_execute then.
 * All calls on one GPU share that GPU's array.  Nothing in it has to start at zero (every partial slab and
 * intermediate is written in full before it is read), so nothing is cleared, and what the last call left there
 * is overwritten.  Two calls that overlap in time on one GPU (different streams, or different threads) race on it:
 * serialise them on one stream. */
int tr_execute_static(eg_graph *g, eg_relation *const *inputs, int n_inputs,
                      eg_relation *const *outputs, int n_outputs, void *hip_stream);

/* Size in bytes of the library's static workspace (the limit of tr_execute_static). */
size_t tr_static_workspace_bytes(void);

/* The aggregation operator of Section 4.2 on its own: out[e] = (+)_{a = 0 .. n_agg-1} partials[a][e],
 * reduced sequentially in ascending a in fp32, then cast once to out's dtype.  partials: device,
 * fp32, slab-major [n_agg][slab_elems] where a slab is the dense row-major tensor of out's bound.
 * out may be strided.  oplus is SUM or MAX.  Also called inside tr_execute. */
int tr_aggregate(eg_agg oplus, const void *partials, int64_t n_agg, int64_t slab_elems,
                 eg_relation *out, void *hip_stream);

/* Fusion across vertices.  Section 3 of the paper writes softmax as four EinSums (row maximum, exp(x - maximum),
 * row sum, division); when such a chain reduces over its last label, that label is not partitioned, all its
 * vertices carry the same partitioning vector and the intermediate tensors have no other consumer, tr_execute
 * runs it as one pass over the rows (the preceding alpha * x + y vertex included when it feeds only the chain),
 * rounding where the separate vertices would have rounded.  Row maxima and sums that other vertices consume are
 * still written.  Up to four element-wise vertices behind the division join the pass as well when their operands are
 * the chain's own values (its source, row maximum, exponentials, row sum, quotient), earlier such vertices, or at most
 * two tensors of the result's shape that exist before the pass runs (the log-probabilities and the cross-entropy
 * gradient of a training step); each is evaluated and rounded as its own vertex would, and only those that something
 * outside the pass reads, or that are outputs, are written.  The pass is reported at the division's vertex.
 * Enabled by default; enable = 0 makes every vertex run on its own.  Changes the workspace size. */
int tr_set_fusion(eg_graph *g, int enable);

/* The alternative to the two-stage path, for comparison (off by default: the method of Section 4.3 is join, then
 * aggregation).  With enable != 0 a contraction whose contracted labels are partitioned runs the join tuples that
 * share an output block as one kernel call that reduces over all their blocks in registers: no partial blocks are
 * written, no aggregation launch follows, and the floating-point summation order is that of the unpartitioned
 * contraction.  Other vertices are not affected.  Changes the workspace size. */
int tr_set_fused_aggregation(eg_graph *g, int enable);

/* How a contraction on the direct-to-LDS kernel lays out the fp32 partial blocks that the aggregation stage sums (Section
 * 4.3's two stages, unchanged).  enable != 0 (the default): when the vertex's blocks are whole output tiles of that kernel,
 * a partial slab holds the tiles one after the other, each in the order the kernel's accumulators lie in registers, and
 * the aggregation kernel that follows undoes the order; same workspace size, same sums in the same order, results equal
 * bit for bit.  enable = 0: every slab is the dense row-major tensor (what tr_aggregate takes).  For comparisons and
 * tests.  Takes effect at the next tr_execute. */
int tr_set_tiled_partials(eg_graph *g, int enable);

/* Another alternative for comparison, off by default.  Section 3 writes attention as a contraction Q x K^T over the head
 * dimension, the softmax chain over the key label (with alpha * x + mask in front when the graph has it) and a second
 * contraction with V over the key label.  With enable != 0 (and tr_set_fusion on) tr_execute runs such a group as one
 * kernel per graph execution, reported at the second contraction's vertex: the scores, exponentials and probabilities are
 * never stored.  Conditions: the group's intermediate tensors have no consumer outside it and are no outputs; neither
 * the head dimension nor the key label is partitioned at the two contractions (other labels may be: the pass covers all
 * their blocks); Q, K, V and the exponentials' vertex are bf16, the row statistics fp32; the head dimension is 32, 64 or
 * 128 and contiguous in Q, K, V and the result; at most two batch labels; the added operand carries only the query and
 * key labels.  Groups that do not qualify run as without this setting, except that non-contiguous head dimensions
 * of bound relations are reported by tr_execute as EG_ERR_LIMIT.
 * Arithmetic: scores and alpha * x + mask are rounded to their vertices' dtypes and the exponentials to bf16, as the
 * separate vertices do; the maximum a row's exponentials are taken against is the running one (rescaled as it grows),
 * and the division by the row sum is applied to the fp32 result of the second contraction instead of to bf16-rounded
 * probabilities, so results differ from the separate vertices' by a few bf16 units in the last place.  A query row whose
 * scores are all -inf gives NaN, as the separate vertices do.  Changes the workspace size. */
int tr_set_fused_attention(eg_graph *g, int enable);

/* Which variant of the block-contraction kernel the (x) = multiply, (+) = sum vertices of this graph run on, for
 * comparisons and for tests that must reach every variant at sizes the library would route elsewhere; results are
 * the same up to summation order.  kernel: 0 = the library chooses per vertex, 1 = the register-staged kernel,
 * 2 = the direct-to-LDS kernel wherever the operand layout allows it.  tile_m x tile_n: 0 x 0 = the library chooses;
 * 128 x 128, 256 x 128 or 256 x 256 = output tile of the direct-to-LDS kernel (fp32 operands have no 256 x 128 variant
 * and take 256 x 256 instead).  waves: 0 = the library chooses, 4 or 8 = waves per workgroup of the 256 x 256 variant.
 * Other values: EG_ERR_LIMIT.  Takes effect at the next tr_execute; changes no workspace size. */
int tr_set_contract_variant(eg_graph *g, int kernel, int tile_m, int tile_n, int waves);

/* ---- Timing of the launches inside tr_execute (for roofline reports) ----------------------------------- */

/* max_launches > 0: from now on tr_execute brackets every kernel launch with a pair of HIP events recorded
 * on its stream, appending to a log that holds up to max_launches launches (later ones are not recorded).
 * The events are created here, never inside tr_execute.  max_launches = 0 switches recording off. */
int tr_profile_enable(eg_graph *g, int max_launches);

/* Forgets the recorded launches (the events are kept for reuse). */
int tr_profile_reset(eg_graph *g);

/* Number of launches recorded since the last reset, or a negative status. */
int tr_profile_count(eg_graph *g);

/* Recorded launch i: its vertex, whether it was the join kernel (0) or the aggregation (1), its
 * eg_kernel_kind (for the aggregation EG_KERNEL_NONE, or EG_KERNEL_AGGREGATE_TILES) and elapsed milliseconds.  The caller must have
 * synchronised the stream.  Host outputs, any may be NULL. */
int tr_profile_get(eg_graph *g, int i, int *vertex, int *stage, int *kernel, float *ms);

/* Recorded launch i: the number of fp32 partial slabs it wrote (a join kernel whose vertex has a partitioned aggregated
 * label, or whose reduction the execution cut further) or read (an aggregation); 0 for a join kernel that wrote its
 * vertex's tensor directly.  With the vertex's bound this gives the bytes the launch moved.  *slabs: host. */
int tr_profile_get_slabs(eg_graph *g, int i, int64_t *slabs);

/* ---- Choosing the partitioning vectors: EinDecomp (Sections 6-8 of the paper) ------------------------------
 *
 * Host-only integer code.  A cost is an upper bound on the floating point numbers that would travel between
 * processors if every join result ran on its own processor (Section 7); on one GPU it is the planner's objective,
 * not a measured quantity.  All pointers are host pointers. */

/* Section 7, "transferring into the join": p (n_X + n_Y), p = prod d = the number of join results, n_X / n_Y the
 * elements of one block of X / Y under d (a vertex with one input pays p n_X).  d: one entry per unique label in
 * schema order, each dividing its label's bound (EG_ERR_BAD_PARTITION / EG_ERR_INDIVISIBLE otherwise). */
int eg_cost_join(const eg_graph *g, int vertex, const int32_t *d, int n_unique_labels, int64_t *cost);

/* Section 7, "transferring into the aggregation": (p / n_agg)(n_agg - 1) n_Z with n_agg = prod d over the
 * aggregated labels and n_Z the elements of one output block. */
int eg_cost_agg(const eg_graph *g, int vertex, const int32_t *d, int n_unique_labels, int64_t *cost);

/* Section 7, "re-partitioning across operations": a tensor with the given bound produced in blocks cut d_producer
 * ways per dimension and consumed in blocks cut d_consumer ways: (n_c/n_int - 1)(n/n_c)(n_c + n_p), plus n_p n/n_c
 * when n_p != n_int.  Zero when the cuts agree.  Every cut entry must divide its bound; should the formula's
 * value not be a whole number the call fails with EG_ERR_BAD_PARTITION. */
int eg_cost_repart(int rank, const int64_t *bound, const int32_t *d_consumer, const int32_t *d_producer, int64_t *cost);

/* Section 8.1: the partitioning vectors of a vertex with exactly p join results whose entries are powers of two
 * dividing the bounds.  *count receives how many there are; the first min(count, capacity) are written to d_out
 * (capacity x n_unique_labels entries, may be NULL), exponents in lexicographic order over the schema.
 * p must be a power of two. */
int eindecomp_viable(const eg_graph *g, int vertex, int p, int32_t *d_out, int capacity, int *count);

/* Sections 8.2-8.4: labels every einsum vertex of the graph with a partitioning vector of p join results (fewer
 * for a vertex whose bounds admit no such vector), as einsum_graph_set_partition would.  When no intermediate
 * result has two consumers the labelling minimises the total cost (dynamic programme over the table M[v, d_Z];
 * *exact = 1).  Otherwise the graph is cut into paths, longest first, each optimised on its own with inputs from
 * outside the path free of charge (*exact = 0).  *total_cost receives the cost of the labelling with every
 * producer -> consumer edge included.  total_cost and exact may be NULL.  On error no vertex is relabelled. */
int eindecomp_plan(eg_graph *g, int p, int64_t *total_cost, int *exact);

/* Cost of the graph's current labelling, split into its three parts (any pointer may be NULL). */
int eindecomp_labelling_cost(const eg_graph *g, int64_t *join, int64_t *agg, int64_t *repart);

/* ---- Measured ceilings of the machine (context for roofline reports; not part of the einsum path) ------- */

/* Enqueues a register-resident loop of bf16 32x32x16 MFMAs (no memory traffic): `waves_per_simd` (1 or 2)
 * waves on each SIMD of `cus` compute units, iters*8 MFMAs per wave.  sink: device, >= 4 bytes, never
 * written.  *flops (host) receives the launch's operation count; the caller times it. */
int eg_ceiling_mfma_bf16(void *sink, int cus, int waves_per_simd, int iters, double *flops, void *hip_stream);

/* The same loop on pseudo-random bf16 operands (sign and mantissa bits from a hash, four A and four B fragments
 * per lane): one wave on each SIMD of `cus` compute units, iters*16 MFMAs per wave.  The chip's clock under the
 * matrix pipes' power draw depends on how many operand bits toggle, so this, not the loop on constants, is the rate
 * a contraction on real data can be held against.  sink, *flops: as above. */
int eg_ceiling_mfma_bf16_random(void *sink, int cus, int iters, double *flops, void *hip_stream);

/* Enqueues a register-resident loop of fp32 subtract + fused-multiply-add pairs (the instruction pair of the
 * squared-distance kernel): `waves_per_simd` (1, 2 or 4) waves on each SIMD of `cus` compute units, iters*64 pairs
 * per lane.  sink: device, >= 4 bytes, never written.  *pairs (host) receives the launch's pair count. */
int eg_ceiling_valu_f32(void *sink, int cus, int waves_per_simd, int iters, double *pairs, void *hip_stream);

/* Enqueues a plain device-to-device copy of `bytes` (multiple of 16; dst/src device, 16-byte aligned). */
int eg_ceiling_copy(void *dst, const void *src, int64_t bytes, void *hip_stream);

/* Enqueues a read-mostly stream with the traffic shape of an aggregation of partial slabs (Section 4.3's second stage):
 * `streams` (2, 8 or 16) consecutive pieces of `bytes` each are read from src, combined without arithmetic and written
 * as one piece of `bytes` to dst (bytes: multiple of 16; dst/src device, 16-byte aligned; src holds streams * bytes). */
int eg_ceiling_read(void *dst, const void *src, int streams, int64_t bytes, void *hip_stream);

/* Message for the last error on this thread (host, valid until the next failing call on the thread). */
const char *eg_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* EINDECOMP_H */
