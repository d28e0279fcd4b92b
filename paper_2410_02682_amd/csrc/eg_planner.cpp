// EinDecomp on the host: the cost model of Section 7 of the paper, the enumeration of partitioning vectors of
// Section 8.1, the dynamic programme of Sections 8.2-8.3 and the path decomposition of Section 8.4.  Pure
// integer code; it only chooses the partitioning vectors that the execution path is otherwise handed.
//
// Readings (the paper leaves these open or contradicts itself):
//   * into the join: p (n_X + n_Y) with p = the number of join results of d (the printed example's "8 x" belongs
//     to a d with 16 results); a vertex with one input pays p n_X;
//   * between a producer and a consumer: n_c is the consumer's sub-tensor size under the consumer's cut and n the
//     tensor's element count, which reproduces the printed total of 320;
//   * the recurrence re-partitions from the producer's output cut (the key of M) to d[l_X; l_XY] of the consumer;
//   * entries of d are powers of two that divide the label's bound; a vertex that has no such vector with p join
//     results gets the largest smaller power of two that has one;
//   * ties go to the vector enumerated first: exponents in lexicographic order over the unique labels in
//     first-appearance order; the cheapest output cut entered first wins at a sink;
//   * paths: among the vertices not yet labelled the longest producer -> consumer chain, ties towards smaller
//     vertex ids; only the edges between consecutive vertices of the path are priced while it is optimised.
#include <algorithm>
#include <cstring>
#include <map>
#include <set>

#include "eg_internal.h"

namespace eg {
namespace {

typedef std::vector<int32_t> Cut;      // one entry per schema label of a vertex, or per dimension of a tensor
typedef __int128 Wide;

struct Choice {                        // best way found to produce one output cut of a vertex
    Cut dz;
    Wide cost;
    Cut d;
    int pick[2];                       // per operand: index into the producer's table, -1 when the edge is not priced
};

void enumerate_rec(const Vertex &v, int label, int left, Cut &cur, std::vector<Cut> &out)
{
    const int nl = (int)v.labels.size();
    if (label == nl - 1) {
        const int64_t dd = 1ll << left;
        if (v.lbound[label] % dd) return;
        cur[label] = (int32_t)dd;
        out.push_back(cur);
        return;
    }
    for (int e = 0; e <= left; e++) {
        const int64_t dd = 1ll << e;
        if (v.lbound[label] % dd) continue;
        cur[label] = (int32_t)dd;
        enumerate_rec(v, label + 1, left - e, cur, out);
    }
}

// Section 8.1: all power-of-two vectors with exactly 2^n join results
std::vector<Cut> viable_exact(const Vertex &v, int n)
{
    std::vector<Cut> out;
    Cut cur(v.labels.size(), 1);
    if (!v.labels.empty()) enumerate_rec(v, 0, n, cur, out);
    else if (n == 0) out.push_back(cur);
    return out;
}

std::vector<Cut> viable_or_fewer(const Vertex &v, int n)
{
    for (; n >= 0; n--) {
        std::vector<Cut> out = viable_exact(v, n);
        if (!out.empty()) return out;
    }
    return {};
}

Wide block_elems(const Vertex &v, const std::vector<int> &dims, const Cut &d)
{
    Wide n = 1;
    for (int l : dims) n *= v.lbound[l] / d[l];
    return n;
}

Wide join_results(const Cut &d)
{
    Wide p = 1;
    for (int32_t x : d) p *= x;
    return p;
}

Wide cost_join(const Vertex &v, const Cut &d)
{
    Wide per = block_elems(v, v.lx, d);
    if (v.n_in > 1) per += block_elems(v, v.ly, d);
    return join_results(d) * per;
}

Wide cost_agg(const Vertex &v, const Cut &d)
{
    Wide n_agg = 1;
    for (int l : v.agg) n_agg *= d[l];
    return join_results(d) / n_agg * (n_agg - 1) * block_elems(v, v.lz, d);
}

// false when the two cuts do not nest (the formula's quotient is then not a whole number)
bool cost_repart(const std::vector<int64_t> &bound, const Cut &d_cons, const Cut &d_prod, Wide &cost)
{
    Wide n_p = 1, n_c = 1, n_int = 1, n = 1;
    for (size_t i = 0; i < bound.size(); i++) {
        const int64_t ep = bound[i] / d_prod[i], ec = bound[i] / d_cons[i];
        n_p *= ep;
        n_c *= ec;
        n_int *= std::min(ep, ec);
        n *= bound[i];
    }
    const Wide blocks = n / n_c, num = (n_c - n_int) * blocks * (n_c + n_p);
    if (num % n_int) return false;
    cost = num / n_int;
    if (n_p != n_int) cost += n_p * blocks;
    return true;
}

Cut operand_cut(const std::vector<int> &dims, const Cut &d)
{
    Cut c(dims.size());
    for (size_t i = 0; i < dims.size(); i++) c[i] = d[dims[i]];
    return c;
}

int log2_exact(int p)
{
    int n = 0;
    while ((1 << n) < p) n++;
    return (1 << n) == p ? n : -1;
}

// The table M of Section 8.2 for the vertices in `order` (ascending ids = a topological order).  An operand is
// priced (producer's M + re-partition) only when `edge(producer, consumer)` says so.
template <typename EdgeFn>
int fill_tables(const eg_graph *g, const std::vector<int> &order, int n, EdgeFn edge, std::map<int, std::vector<Choice>> &M)
{
    for (int vi : order) {
        const Vertex &v = g->v[vi];
        std::vector<Choice> table;
        std::map<Cut, int> index;
        const std::vector<Cut> cand = viable_or_fewer(v, n);
        if (cand.empty()) return fail(EG_ERR_BAD_PARTITION, "vertex %d has no partitioning vector", vi);
        for (const Cut &d : cand) {
            Wide c = cost_join(v, d) + cost_agg(v, d);
            int pick[2] = {-1, -1};
            for (int k = 0; k < v.n_in; k++) {
                const int u = v.in[k];
                if (g->v[u].is_input || !edge(u, vi)) continue;
                if (k == 1 && v.in[0] == u) return fail(EG_ERR_LIMIT, "vertex %d takes vertex %d for both operands: not handled by the planner", vi, u);
                const Cut want = operand_cut(k == 0 ? v.lx : v.ly, d);
                const std::vector<Choice> &tu = M[u];
                Wide best = -1;
                for (size_t i = 0; i < tu.size(); i++) {
                    Wide r;
                    if (!cost_repart(g->v[u].bound, want, tu[i].dz, r)) return fail(EG_ERR_BAD_PARTITION, "cuts of vertex %d do not nest", u);
                    const Wide t = tu[i].cost + r;
                    if (best < 0 || t < best) { best = t; pick[k] = (int)i; }
                }
                c += best;
            }
            Cut dz = operand_cut(v.lz, d);
            auto it = index.find(dz);
            if (it == index.end()) {
                index[dz] = (int)table.size();
                table.push_back(Choice{dz, c, d, {pick[0], pick[1]}});
            } else if (c < table[it->second].cost) {
                Choice &ch = table[it->second];
                ch.cost = c; ch.d = d; ch.pick[0] = pick[0]; ch.pick[1] = pick[1];
            }
        }
        M[vi] = std::move(table);
    }
    return EG_OK;
}

void backtrack(const eg_graph *g, const std::map<int, std::vector<Choice>> &M, int vi, int entry, std::map<int, Cut> &labels)
{
    const Choice &ch = M.at(vi)[entry];
    labels[vi] = ch.d;
    const Vertex &v = g->v[vi];
    for (int k = 0; k < v.n_in; k++)
        if (ch.pick[k] >= 0) backtrack(g, M, v.in[k], ch.pick[k], labels);
}

int cheapest(const std::vector<Choice> &t)
{
    int best = 0;
    for (size_t i = 1; i < t.size(); i++)
        if (t[i].cost < t[best].cost) best = (int)i;
    return best;
}

// total cost of a complete labelling, every producer -> consumer edge included
int labelling_cost(const eg_graph *g, const std::map<int, Cut> &labels, Wide &join, Wide &agg, Wide &repart)
{
    join = agg = repart = 0;
    for (size_t vi = 0; vi < g->v.size(); vi++) {
        const Vertex &v = g->v[vi];
        if (v.is_input) continue;
        const Cut &d = labels.at((int)vi);
        join += cost_join(v, d);
        agg += cost_agg(v, d);
        for (int k = 0; k < v.n_in; k++) {
            const int u = v.in[k];
            if (g->v[u].is_input) continue;
            Wide r;
            if (!cost_repart(g->v[u].bound, operand_cut(k == 0 ? v.lx : v.ly, d), operand_cut(g->v[u].lz, labels.at(u)), r))
                return fail(EG_ERR_BAD_PARTITION, "cuts of vertex %d and its consumer %zu do not nest", u, vi);
            repart += r;
        }
    }
    return EG_OK;
}

int to_i64(Wide x, int64_t *out)
{
    if (x < 0 || x > (Wide)INT64_MAX) return fail(EG_ERR_LIMIT, "cost does not fit 63 bits");
    *out = (int64_t)x;
    return EG_OK;
}

int check_vertex(const eg_graph *g, int vertex, const int32_t *d, int n)
{
    if (!g || !d) return fail(EG_ERR_NULL, "NULL argument");
    if (vertex < 0 || vertex >= (int)g->v.size() || g->v[vertex].is_input) return fail(EG_ERR_BAD_VERTEX, "vertex %d is not an einsum vertex", vertex);
    const Vertex &v = g->v[vertex];
    if (n != (int)v.labels.size()) return fail(EG_ERR_BAD_PARTITION, "vertex %d has %zu unique labels, %d entries given", vertex, v.labels.size(), n);
    for (int l = 0; l < n; l++) {
        if (d[l] < 1) return fail(EG_ERR_BAD_PARTITION, "d[%d] = %d must be >= 1", l, d[l]);
        if (v.lbound[l] % d[l]) return fail(EG_ERR_INDIVISIBLE, "label '%c': %d does not divide bound %lld", v.labels[l], d[l], (long long)v.lbound[l]);
    }
    return EG_OK;
}

}  // namespace
}  // namespace eg

using namespace eg;

extern "C" {

int eg_cost_join(const eg_graph *g, int vertex, const int32_t *d, int n_unique_labels, int64_t *cost)
{
    int rc = check_vertex(g, vertex, d, n_unique_labels);
    if (rc) return rc;
    if (!cost) return fail(EG_ERR_NULL, "cost is NULL");
    return to_i64(cost_join(g->v[vertex], Cut(d, d + n_unique_labels)), cost);
}

int eg_cost_agg(const eg_graph *g, int vertex, const int32_t *d, int n_unique_labels, int64_t *cost)
{
    int rc = check_vertex(g, vertex, d, n_unique_labels);
    if (rc) return rc;
    if (!cost) return fail(EG_ERR_NULL, "cost is NULL");
    return to_i64(cost_agg(g->v[vertex], Cut(d, d + n_unique_labels)), cost);
}

int eg_cost_repart(int rank, const int64_t *bound, const int32_t *d_consumer, const int32_t *d_producer, int64_t *cost)
{
    if (rank < 0 || rank > EG_MAX_RANK) return fail(EG_ERR_LIMIT, "rank %d", rank);
    if (rank > 0 && (!bound || !d_consumer || !d_producer)) return fail(EG_ERR_NULL, "NULL argument");
    if (!cost) return fail(EG_ERR_NULL, "cost is NULL");
    for (int i = 0; i < rank; i++) {
        if (bound[i] < 1) return fail(EG_ERR_BAD_BOUND, "bound[%d] = %lld", i, (long long)bound[i]);
        if (d_consumer[i] < 1 || d_producer[i] < 1) return fail(EG_ERR_BAD_PARTITION, "entry %d must be >= 1", i);
        if (bound[i] % d_consumer[i] || bound[i] % d_producer[i]) return fail(EG_ERR_INDIVISIBLE, "entry %d does not divide bound %lld", i, (long long)bound[i]);
    }
    Wide c;
    if (!cost_repart(std::vector<int64_t>(bound, bound + rank), Cut(d_consumer, d_consumer + rank), Cut(d_producer, d_producer + rank), c))
        return fail(EG_ERR_BAD_PARTITION, "the two cuts do not nest");
    return to_i64(c, cost);
}

int eindecomp_viable(const eg_graph *g, int vertex, int p, int32_t *d_out, int capacity, int *count)
{
    if (!g || !count) return fail(EG_ERR_NULL, "NULL argument");
    if (vertex < 0 || vertex >= (int)g->v.size() || g->v[vertex].is_input) return fail(EG_ERR_BAD_VERTEX, "vertex %d is not an einsum vertex", vertex);
    const int n = p >= 1 ? log2_exact(p) : -1;
    if (n < 0 || n > 20) return fail(EG_ERR_BAD_PARTITION, "p = %d must be a power of two up to 2^20", p);
    const Vertex &v = g->v[vertex];
    const std::vector<Cut> all = viable_exact(v, n);
    *count = (int)all.size();
    if (d_out) {
        const size_t nl = v.labels.size();
        for (size_t i = 0; i < all.size() && (int)i < capacity; i++) memcpy(d_out + i * nl, all[i].data(), nl * sizeof(int32_t));
    }
    return EG_OK;
}

int eindecomp_labelling_cost(const eg_graph *g, int64_t *join, int64_t *agg, int64_t *repart)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    std::map<int, Cut> labels;
    for (size_t i = 0; i < g->v.size(); i++)
        if (!g->v[i].is_input) labels[(int)i] = g->v[i].d;
    Wide j, a, r;
    int rc = labelling_cost(g, labels, j, a, r);
    if (rc) return rc;
    int64_t t;
    if (join && (rc = to_i64(j, join))) return rc;
    if (agg && (rc = to_i64(a, agg))) return rc;
    if (repart && (rc = to_i64(r, repart))) return rc;
    return to_i64(j + a + r, &t);
}

int eindecomp_plan(eg_graph *g, int p, int64_t *total_cost, int *exact)
{
    if (!g) return fail(EG_ERR_NULL, "graph is NULL");
    const int n = p >= 1 ? log2_exact(p) : -1;
    if (n < 0 || n > 20) return fail(EG_ERR_BAD_PARTITION, "p = %d must be a power of two up to 2^20", p);
    const int nv = (int)g->v.size();
    std::vector<int> ein;
    std::vector<std::set<int>> consumers(nv);
    for (int i = 0; i < nv; i++) {
        if (g->v[i].is_input) continue;
        ein.push_back(i);
        for (int k = 0; k < g->v[i].n_in; k++) consumers[g->v[i].in[k]].insert(i);
    }
    if (ein.empty()) return fail(EG_ERR_BAD_VERTEX, "the graph has no einsum vertex");
    bool shared = false;
    for (int i : ein) shared = shared || consumers[i].size() > 1;

    std::map<int, Cut> labels;
    if (!shared) {
        // Sections 8.2-8.3: every intermediate result has one consumer, the table describes whole subgraphs
        std::map<int, std::vector<Choice>> M;
        int rc = fill_tables(g, ein, n, [](int, int) { return true; }, M);
        if (rc) return rc;
        for (int i : ein)
            if (consumers[i].empty()) backtrack(g, M, i, cheapest(M[i]), labels);
    } else {
        // Section 8.4: longest path among the vertices still without a label, optimised on its own, and again
        std::set<int> todo(ein.begin(), ein.end());
        while (!todo.empty()) {
            std::map<int, std::vector<int>> best_to;          // longest chain of unlabelled vertices ending at each
            auto better = [](const std::vector<int> &a, const std::vector<int> &b) {   // a before b?
                if (a.size() != b.size()) return a.size() > b.size();
                return a < b;
            };
            std::vector<int> path;
            for (int i : todo) {
                std::vector<int> here{i};
                for (int k = 0; k < g->v[i].n_in; k++) {
                    auto it = best_to.find(g->v[i].in[k]);
                    if (it == best_to.end()) continue;
                    std::vector<int> cand = it->second;
                    cand.push_back(i);
                    if (better(cand, here)) here = cand;
                }
                best_to[i] = here;
                if (path.empty() || better(here, path)) path = here;
            }
            std::set<std::pair<int, int>> edges;
            for (size_t i = 0; i + 1 < path.size(); i++) edges.insert({path[i], path[i + 1]});
            std::map<int, std::vector<Choice>> M;
            int rc = fill_tables(g, path, n, [&](int u, int c) { return edges.count({u, c}) > 0; }, M);
            if (rc) return rc;
            backtrack(g, M, path.back(), cheapest(M[path.back()]), labels);
            for (int i : path) todo.erase(i);
        }
    }
    Wide j, a, r;
    int rc = labelling_cost(g, labels, j, a, r);
    if (rc) return rc;
    int64_t total;
    rc = to_i64(j + a + r, &total);
    if (rc) return rc;
    for (auto &kv : labels) {
        rc = einsum_graph_set_partition(g, kv.first, kv.second.data(), (int)kv.second.size());
        if (rc) return rc;
    }
    if (total_cost) *total_cost = total;
    if (exact) *exact = shared ? 0 : 1;
    return EG_OK;
}

}  // extern "C"
