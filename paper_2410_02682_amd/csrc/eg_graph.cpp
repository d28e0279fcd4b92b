// Host-side EinGraph container, spec parsing, validation and the join planner's integer tables.
//
// Paper passages: the vertex triple (bound, EinSum, inputs) and the partition annotation are Sections
// 5-6; label projection b[l1; l2] and the aggregated-label rule are Section 3; tensor relations and
// block extents b/d are Section 4.1; the join's matching rule and key naming are Section 4.2; the join
// count N = prod d[l_X (.) l_Y] is Section 6 and n_agg = prod d[l_agg] is Section 7.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "eg_internal.h"

namespace eg {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

static thread_local bool g_validate_only = false;
bool validate_only() { return g_validate_only; }
void set_validate_only(bool on) { g_validate_only = on; }

// Parses "ij,jk->ik" / "ij->i" / "bc,bc->" into label characters per operand.
static int parse_spec(const char *spec, std::string &sx, std::string &sy, std::string &sz, bool &binary)
{
    const char *arrow = strstr(spec, "->");
    if (!arrow) return fail(EG_ERR_BAD_SPEC, "spec '%s' has no '->'", spec);
    std::string lhs(spec, arrow - spec);
    sz = std::string(arrow + 2);
    size_t comma = lhs.find(',');
    if (comma == std::string::npos) {
        binary = false;
        sx = lhs;
        sy.clear();
    } else {
        binary = true;
        sx = lhs.substr(0, comma);
        sy = lhs.substr(comma + 1);
        if (sy.find(',') != std::string::npos) return fail(EG_ERR_BAD_SPEC, "spec '%s': an EinSum is unary or binary", spec);
    }
    auto ok = [](const std::string &s) {
        for (char c : s)
            if (!((c >= 'a' && c <= 'z') || (c >= 'A' && c <= 'Z'))) return false;
        return true;
    };
    if (!ok(sx) || !ok(sy) || !ok(sz)) return fail(EG_ERR_BAD_SPEC, "spec '%s': labels are single letters", spec);
    if (sx.empty()) return fail(EG_ERR_BAD_SPEC, "spec '%s': first operand has no labels", spec);
    if (binary && sy.empty()) return fail(EG_ERR_BAD_SPEC, "spec '%s': second operand has no labels", spec);
    if (sx.size() > EG_MAX_RANK || sy.size() > EG_MAX_RANK || sz.size() > EG_MAX_RANK)
        return fail(EG_ERR_LIMIT, "spec '%s': rank above %d", spec, EG_MAX_RANK);
    return EG_OK;
}

static bool has_repeat(const std::string &s)
{
    for (size_t i = 0; i < s.size(); i++)
        for (size_t j = i + 1; j < s.size(); j++)
            if (s[i] == s[j]) return true;
    return false;
}

// Builds the tuple table of a vertex for its current d.
static void build_plan(Vertex &v)
{
    Plan &p = v.plan;
    const int nl = (int)v.labels.size();
    p = Plan();
    p.n_tuples = 1;
    for (int l = 0; l < nl; l++) p.n_tuples *= v.d[l];
    p.n_agg = 1;
    for (int a : v.agg) p.n_agg *= v.d[a];
    p.n_groups = p.n_tuples / p.n_agg;

    // dense row-major strides of X, Y, Z per dimension
    auto dense = [&](const std::vector<int> &labs) {
        std::vector<int64_t> st(labs.size());
        int64_t acc = 1;
        for (int i = (int)labs.size() - 1; i >= 0; i--) {
            st[i] = acc;
            acc *= v.lbound[labs[i]];
        }
        return st;
    };
    std::vector<int64_t> stx = dense(v.lx), sty = dense(v.ly), stz = dense(v.lz);

    const int64_t N = p.n_tuples;
    p.key.resize(N * nl);
    p.key_x.resize(N * v.lx.size());
    p.key_y.resize(N * v.ly.size());
    p.key_z.resize(N * v.lz.size());
    p.agg_idx.resize(N);
    p.group.resize(N);
    p.off_x.resize(N);
    p.off_y.resize(N);
    p.off_z.resize(N);
    std::vector<int32_t> key(nl, 0);
    for (int64_t t = 0; t < N; t++) {
        // row-major over I(d) on the schema, last label fastest
        int64_t rem = t;
        for (int l = nl - 1; l >= 0; l--) {
            key[l] = (int32_t)(rem % v.d[l]);
            rem /= v.d[l];
        }
        for (int l = 0; l < nl; l++) p.key[t * nl + l] = key[l];
        int64_t ox = 0, oy = 0, oz = 0;
        for (size_t i = 0; i < v.lx.size(); i++) {
            int l = v.lx[i];
            p.key_x[t * v.lx.size() + i] = key[l];
            ox += (int64_t)key[l] * (v.lbound[l] / v.d[l]) * stx[i];
        }
        for (size_t i = 0; i < v.ly.size(); i++) {
            int l = v.ly[i];
            p.key_y[t * v.ly.size() + i] = key[l];
            oy += (int64_t)key[l] * (v.lbound[l] / v.d[l]) * sty[i];
        }
        int64_t grp = 0;
        for (size_t i = 0; i < v.lz.size(); i++) {
            int l = v.lz[i];
            p.key_z[t * v.lz.size() + i] = key[l];
            oz += (int64_t)key[l] * (v.lbound[l] / v.d[l]) * stz[i];
            grp = grp * v.d[l] + key[l];
        }
        int64_t ai = 0;
        for (int a : v.agg) ai = ai * v.d[a] + key[a];
        p.agg_idx[t] = (int32_t)ai;
        p.group[t] = (int32_t)grp;
        p.off_x[t] = ox;
        p.off_y[t] = oy;
        p.off_z[t] = oz;
    }
    p.valid = true;
}

}  // namespace eg

using namespace eg;

extern "C" {

const char *eg_last_error(void) { return g_err; }

int einsum_graph_create(eg_graph **g)
{
    if (!g) return fail(EG_ERR_NULL, "einsum_graph_create: g is NULL");
    *g = new eg_graph();
    return EG_OK;
}

void einsum_graph_destroy(eg_graph *g)
{
    if (!g) return;
    eg_release_events(g);
    delete g;
}

int einsum_graph_num_vertices(const eg_graph *g)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    return (int)g->v.size();
}

int einsum_graph_add_input(eg_graph *g, int rank, const int64_t *bound, eg_dtype dtype, int *vertex)
{
    if (!g || (rank > 0 && !bound)) return fail(EG_ERR_NULL, "einsum_graph_add_input: NULL argument");
    if (rank < 0 || rank > EG_MAX_RANK) return fail(EG_ERR_LIMIT, "rank %d outside 0..%d", rank, EG_MAX_RANK);
    if (dtype != EG_F32 && dtype != EG_BF16) return fail(EG_ERR_DTYPE, "unknown dtype %d", (int)dtype);
    Vertex v;
    v.is_input = true;
    v.dtype = dtype;
    for (int i = 0; i < rank; i++) {
        if (bound[i] < 1) return fail(EG_ERR_BAD_BOUND, "bound[%d] = %lld must be >= 1", i, (long long)bound[i]);
        v.bound.push_back(bound[i]);
    }
    g->v.push_back(v);
    g->inputs.push_back((int)g->v.size() - 1);
    if (vertex) *vertex = (int)g->v.size() - 1;
    return EG_OK;
}

int einsum_graph_add_einsum(eg_graph *g, const char *spec, eg_join otimes, eg_agg oplus, double alpha,
                            const int *inputs, int n_inputs, eg_dtype out_dtype, int *vertex)
{
    if (!g || !spec || !inputs) return fail(EG_ERR_NULL, "einsum_graph_add_einsum: NULL argument");
    if (out_dtype != EG_F32 && out_dtype != EG_BF16) return fail(EG_ERR_DTYPE, "unknown dtype %d", (int)out_dtype);
    std::string sx, sy, sz;
    bool binary;
    int rc = parse_spec(spec, sx, sy, sz, binary);
    if (rc) return rc;
    if (n_inputs != (binary ? 2 : 1))
        return fail(EG_ERR_BAD_SPEC, "spec '%s' names %d operands but %d inputs were given", spec, binary ? 2 : 1, n_inputs);
    const bool unary_op = (int)otimes >= 32;
    switch ((int)otimes) {
    case EG_MUL: case EG_ADD: case EG_SUB: case EG_DIV: case EG_SQDIFF: case EG_ABSDIFF: case EG_EXP_SUB:
    case EG_RELU_GRAD: case EG_SILU_MUL: case EG_IDENT: case EG_SCALE: case EG_RELU: case EG_EXP: case EG_LOG: break;
    default: return fail(EG_ERR_BAD_OP, "unknown scalar function %d", (int)otimes);
    }
    if (unary_op == binary)
        return fail(EG_ERR_BAD_OP, "scalar function %d is %s but the spec '%s' is %s", (int)otimes,
                    unary_op ? "unary" : "binary", spec, binary ? "binary" : "unary");
    if (has_repeat(sx) || has_repeat(sy) || has_repeat(sz))
        return fail(EG_ERR_REPEATED_LABEL, "spec '%s': a label is repeated inside one operand", spec);
    for (int i = 0; i < n_inputs; i++)
        if (inputs[i] < 0 || inputs[i] >= (int)g->v.size())
            return fail(EG_ERR_BAD_VERTEX, "input vertex %d does not exist yet", inputs[i]);

    Vertex v;
    v.spec = spec;
    v.dtype = out_dtype;
    v.otimes = (int)otimes;
    v.oplus = (int)oplus;
    v.alpha = alpha;
    v.n_in = n_inputs;
    v.in[0] = inputs[0];
    v.in[1] = binary ? inputs[1] : -1;
    // schema: unique labels in first-appearance order over l_X then l_Y
    auto schema_index = [&](char c) {
        for (size_t i = 0; i < v.labels.size(); i++)
            if (v.labels[i] == c) return (int)i;
        return -1;
    };
    const Vertex &vx = g->v[inputs[0]];
    if (vx.bound.size() != sx.size())
        return fail(EG_ERR_BAD_BOUND, "spec '%s': first operand has %zu labels but its tensor has rank %zu", spec, sx.size(), vx.bound.size());
    for (size_t i = 0; i < sx.size(); i++) {
        v.labels.push_back(sx[i]);
        v.lbound.push_back(vx.bound[i]);
        v.lx.push_back((int)v.labels.size() - 1);
    }
    if (binary) {
        const Vertex &vy = g->v[inputs[1]];
        if (vy.bound.size() != sy.size())
            return fail(EG_ERR_BAD_BOUND, "spec '%s': second operand has %zu labels but its tensor has rank %zu", spec, sy.size(), vy.bound.size());
        for (size_t i = 0; i < sy.size(); i++) {
            int l = schema_index(sy[i]);
            if (l < 0) {
                v.labels.push_back(sy[i]);
                v.lbound.push_back(vy.bound[i]);
                l = (int)v.labels.size() - 1;
            } else if (v.lbound[l] != vy.bound[i]) {
                return fail(EG_ERR_BAD_BOUND, "spec '%s': label '%c' has bounds %lld and %lld", spec, sy[i],
                            (long long)v.lbound[l], (long long)vy.bound[i]);
            }
            v.ly.push_back(l);
        }
    }
    if (v.labels.size() > EG_MAX_LABELS) return fail(EG_ERR_LIMIT, "spec '%s': more than %d unique labels", spec, EG_MAX_LABELS);
    for (char c : sz) {
        int l = schema_index(c);
        if (l < 0) return fail(EG_ERR_BROADCAST, "spec '%s': output label '%c' occurs in no input (broadcast)", spec, c);
        v.lz.push_back(l);
        v.bound.push_back(v.lbound[l]);
    }
    for (size_t l = 0; l < v.labels.size(); l++)
        if (sz.find(v.labels[l]) == std::string::npos) v.agg.push_back((int)l);
    if (!v.agg.empty() && oplus != EG_AGG_SUM && oplus != EG_AGG_MAX)
        return fail(EG_ERR_BAD_OP, "spec '%s' aggregates a label but no aggregation operator was given", spec);
    if (v.agg.empty()) v.oplus = EG_AGG_NONE;
    v.d.assign(v.labels.size(), 1);
    build_plan(v);
    g->v.push_back(v);
    if (vertex) *vertex = (int)g->v.size() - 1;
    return EG_OK;
}

int einsum_graph_set_partition(eg_graph *g, int vertex, const int32_t *d, int n_unique_labels)
{
    if (!g || !d) return fail(EG_ERR_NULL, "einsum_graph_set_partition: NULL argument");
    if (vertex < 0 || vertex >= (int)g->v.size() || g->v[vertex].is_input)
        return fail(EG_ERR_BAD_VERTEX, "vertex %d is not an einsum vertex", vertex);
    Vertex &v = g->v[vertex];
    if (n_unique_labels != (int)v.labels.size())
        return fail(EG_ERR_BAD_PARTITION, "vertex %d has %zu unique labels, %d partition entries given", vertex, v.labels.size(), n_unique_labels);
    int64_t tuples = 1;
    for (int l = 0; l < n_unique_labels; l++) {
        if (d[l] < 1) return fail(EG_ERR_BAD_PARTITION, "d[%d] = %d must be >= 1", l, d[l]);
        if (v.lbound[l] % d[l]) return fail(EG_ERR_INDIVISIBLE, "label '%c': %d does not divide bound %lld", v.labels[l], d[l], (long long)v.lbound[l]);
        tuples *= d[l];
        if (tuples > (1 << 20)) return fail(EG_ERR_LIMIT, "more than 2^20 join tuples");
    }
    v.d.assign(d, d + n_unique_labels);
    build_plan(v);
    return EG_OK;
}

int einsum_graph_mark_output(eg_graph *g, int vertex)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    if (vertex < 0 || vertex >= (int)g->v.size() || g->v[vertex].is_input)
        return fail(EG_ERR_BAD_VERTEX, "vertex %d is not an einsum vertex", vertex);
    if (!g->v[vertex].is_output) {
        g->v[vertex].is_output = true;
        g->outputs.push_back(vertex);
    }
    return EG_OK;
}

int einsum_graph_plan(eg_graph *g, int vertex, eg_plan_view *out)
{
    if (!g || !out) return fail(EG_ERR_NULL, "einsum_graph_plan: NULL argument");
    if (vertex < 0 || vertex >= (int)g->v.size() || g->v[vertex].is_input)
        return fail(EG_ERR_BAD_VERTEX, "vertex %d is not an einsum vertex", vertex);
    Vertex &v = g->v[vertex];
    if (!v.plan.valid) build_plan(v);
    memset(out, 0, sizeof *out);
    out->n_labels = (int32_t)v.labels.size();
    for (size_t l = 0; l < v.labels.size(); l++) {
        out->labels[l] = v.labels[l];
        out->bound[l] = v.lbound[l];
        out->d[l] = v.d[l];
    }
    out->rank_x = (int32_t)v.lx.size();
    out->rank_y = (int32_t)v.ly.size();
    out->rank_z = (int32_t)v.lz.size();
    for (size_t i = 0; i < v.lx.size(); i++) { out->d_x[i] = v.d[v.lx[i]]; out->block_x[i] = v.lbound[v.lx[i]] / v.d[v.lx[i]]; }
    for (size_t i = 0; i < v.ly.size(); i++) { out->d_y[i] = v.d[v.ly[i]]; out->block_y[i] = v.lbound[v.ly[i]] / v.d[v.ly[i]]; }
    for (size_t i = 0; i < v.lz.size(); i++) {
        out->d_z[i] = v.d[v.lz[i]];
        out->block_z[i] = v.lbound[v.lz[i]] / v.d[v.lz[i]];
        out->bound_z[i] = v.lbound[v.lz[i]];
    }
    out->n_tuples = v.plan.n_tuples;
    out->n_agg = v.plan.n_agg;
    out->n_groups = v.plan.n_groups;
    out->kernel = eg_route_vertex(g, vertex);
    // repartition between vertices (Section 5): the producer's output partitioning against what this
    // vertex needs for the operand.  Graph inputs are bound at execution time and are not counted here.
    auto differs = [&](int producer, const std::vector<int> &labs) {
        const Vertex &pv = g->v[producer];
        if (pv.is_input) return 0;
        for (size_t i = 0; i < labs.size(); i++)
            if (pv.d[pv.lz[i]] != v.d[labs[i]]) return 1;
        return 0;
    };
    out->repart_x = differs(v.in[0], v.lx);
    out->repart_y = v.n_in > 1 ? differs(v.in[1], v.ly) : 0;
    out->key = v.plan.key.data();
    out->key_x = v.plan.key_x.data();
    out->key_y = v.plan.key_y.data();
    out->key_z = v.plan.key_z.data();
    out->agg_idx = v.plan.agg_idx.data();
    out->group = v.plan.group.data();
    out->off_x = v.plan.off_x.data();
    out->off_y = v.plan.off_y.data();
    out->off_z = v.plan.off_z.data();
    return EG_OK;
}

// ---------------------------------------------------------------------------------------- relations
int tensor_partition(void *dev_ptr, eg_dtype dtype, int rank, const int64_t *bound,
                     const int64_t *strides_or_null, const int32_t *d, eg_relation **rel)
{
    if (!dev_ptr || !rel || (rank > 0 && (!bound || !d))) return fail(EG_ERR_NULL, "tensor_partition: NULL argument");
    if (rank < 0 || rank > EG_MAX_RANK) return fail(EG_ERR_LIMIT, "rank %d outside 0..%d", rank, EG_MAX_RANK);
    if (dtype != EG_F32 && dtype != EG_BF16) return fail(EG_ERR_DTYPE, "unknown dtype %d", (int)dtype);
    eg_relation *r = new eg_relation();
    r->ptr = dev_ptr;
    r->dtype = dtype;
    int64_t acc = 1;
    r->stride.assign(rank, 0);
    for (int i = rank - 1; i >= 0; i--) {
        if (bound[i] < 1) { delete r; return fail(EG_ERR_BAD_BOUND, "bound[%d] = %lld must be >= 1", i, (long long)bound[i]); }
        if (d[i] < 1) { delete r; return fail(EG_ERR_BAD_PARTITION, "d[%d] = %d must be >= 1", i, d[i]); }
        if (bound[i] % d[i]) { delete r; return fail(EG_ERR_INDIVISIBLE, "d[%d] = %d does not divide bound %lld", i, d[i], (long long)bound[i]); }
        r->stride[i] = strides_or_null ? strides_or_null[i] : acc;
        if (strides_or_null && strides_or_null[i] < 0) { delete r; return fail(EG_ERR_BAD_BOUND, "negative strides are not supported"); }
        acc *= bound[i];
    }
    r->bound.assign(bound, bound + rank);
    r->d.assign(d, d + rank);
    *rel = r;
    return EG_OK;
}

int tensor_relation_block(const eg_relation *rel, const int32_t *key, int64_t *offset, int64_t *bound, int64_t *strides)
{
    if (!rel || (!key && !rel->bound.empty())) return fail(EG_ERR_NULL, "tensor_relation_block: NULL argument");
    int64_t off = 0;
    for (size_t i = 0; i < rel->bound.size(); i++) {
        if (key[i] < 0 || key[i] >= rel->d[i]) return fail(EG_ERR_BAD_PARTITION, "key[%zu] = %d outside 0..%d", i, key[i], rel->d[i] - 1);
        int64_t e = rel->bound[i] / rel->d[i];
        off += (int64_t)key[i] * e * rel->stride[i];
        if (bound) bound[i] = e;
        if (strides) strides[i] = rel->stride[i];
    }
    if (offset) *offset = off;
    return EG_OK;
}

void tensor_relation_destroy(eg_relation *rel) { delete rel; }

}  // extern "C"
