// Host-side layout builder: validates a batch of DAGs and produces what the
// level-synchronous sweeps need: parent and child CSR, longest-path levels in both
// directions, and per-graph level buckets.
//
// Section 2 of the paper models a network as a DAG whose ops receive tensors from their
// parent ops; the message passing of Section 2.2 step 2 runs in two directions, one starting
// at the nodes without parents and one starting at the nodes without children.  A node's
// level is the length of the longest path from a root (top-down) or to a leaf (bottom-up), so
// every neighbour a node aggregates over sits on a strictly lower level and is final before
// the node is visited.
#include <algorithm>
#include <cstdint>
#include <numeric>
#include <string>
#include <vector>

#include "internal.h"

namespace pl {

namespace {

// Counting-sort one direction's CSR for graph-local edges (key -> list of values).
void fill_csr(int32_t n, int32_t m, const int32_t *key, const int32_t *val, int64_t base_ptr,
              int64_t *ptr /* n+1 entries, absolute */, int32_t *idx /* m entries */)
{
    std::vector<int32_t> cnt(static_cast<size_t>(n) + 1, 0);
    for (int32_t e = 0; e < m; ++e) cnt[key[e] + 1]++;
    for (int32_t v = 0; v < n; ++v) cnt[v + 1] += cnt[v];
    for (int32_t v = 0; v <= n; ++v) ptr[v] = base_ptr + cnt[v];
    std::vector<int32_t> cursor(cnt.begin(), cnt.end() - 1);
    for (int32_t e = 0; e < m; ++e) idx[cursor[key[e]]++] = val[e];
    for (int32_t v = 0; v < n; ++v) std::sort(idx + cnt[v], idx + cnt[v + 1]);
}

// Longest-path levels over `nbr` (the lists a node waits for).  `rev` are the opposite
// lists.  Returns false if some node is never released, i.e. the graph has a cycle.
bool longest_path_levels(int32_t n, const int64_t *nbr_ptr, const int64_t *rev_ptr,
                         const int32_t *rev_idx, int64_t base, int32_t *level)
{
    std::vector<int32_t> waiting(n), queue;
    queue.reserve(n);
    for (int32_t v = 0; v < n; ++v) {
        waiting[v] = static_cast<int32_t>(nbr_ptr[v + 1] - nbr_ptr[v]);
        level[v] = 0;
        if (waiting[v] == 0) queue.push_back(v);
    }
    for (size_t head = 0; head < queue.size(); ++head) {
        const int32_t u = queue[head];
        for (int64_t p = rev_ptr[u] - base; p < rev_ptr[u + 1] - base; ++p) {
            const int32_t c = rev_idx[p];
            level[c] = std::max(level[c], level[u] + 1);
            if (--waiting[c] == 0) queue.push_back(c);
        }
    }
    return static_cast<int32_t>(queue.size()) == n;
}

// Bucket nodes by level, ascending id inside a level; lvl_ptr gets depth+1 positions.
void bucket_by_level(int32_t n, int32_t depth, const int32_t *level, int32_t *order,
                     int32_t *lvl_ptr)
{
    std::fill(lvl_ptr, lvl_ptr + depth + 1, 0);
    for (int32_t v = 0; v < n; ++v) lvl_ptr[level[v] + 1]++;
    for (int32_t l = 0; l < depth; ++l) lvl_ptr[l + 1] += lvl_ptr[l];
    std::vector<int32_t> cursor(lvl_ptr, lvl_ptr + depth);
    for (int32_t v = 0; v < n; ++v) order[cursor[level[v]]++] = v;
}

}  // namespace

int build_layout(int32_t B, const int32_t *n_nodes, const int32_t *n_edges,
                 const int32_t *edge_src, const int32_t *edge_dst, HostLayout *out)
{
    HostLayout &L = *out;
    L = HostLayout();
    L.B = B;
    L.node_off.assign(static_cast<size_t>(B) + 1, 0);
    L.edge_off.assign(static_cast<size_t>(B) + 1, 0);
    for (int32_t b = 0; b < B; ++b) {
        if (n_nodes[b] < 1)
            return fail(PL_ERR_SHAPE, "graph " + std::to_string(b) + " has no nodes");
        if (n_edges[b] < 0)
            return fail(PL_ERR_SHAPE, "graph " + std::to_string(b) + " has a negative edge count");
        L.node_off[b + 1] = L.node_off[b] + n_nodes[b];
        L.edge_off[b + 1] = L.edge_off[b] + n_edges[b];
    }
    L.n_tot = L.node_off[B];
    L.e_tot = L.edge_off[B];
    if (L.n_tot > INT32_MAX / 2 || L.e_tot > INT32_MAX / 2)
        return fail(PL_ERR_SHAPE, "batch too large for 32-bit device indices");
    if (L.e_tot > 0 && (!edge_src || !edge_dst)) return fail(PL_ERR_NULL, "edge arrays are NULL");

    L.par_ptr.assign(L.n_tot + 1, 0);
    L.chi_ptr.assign(L.n_tot + 1, 0);
    L.par_idx.resize(L.e_tot);
    L.chi_idx.resize(L.e_tot);
    L.td_level.resize(L.n_tot);
    L.bu_level.resize(L.n_tot);
    L.td_order.resize(L.n_tot);
    L.bu_order.resize(L.n_tot);
    L.depth.resize(B);
    L.lvl_off.assign(static_cast<size_t>(B) + 1, 0);

    for (int32_t b = 0; b < B; ++b) {
        const int32_t n = n_nodes[b], m = n_edges[b];
        const int64_t n0 = L.node_off[b], e0 = L.edge_off[b];
        const int32_t *src = edge_src + e0, *dst = edge_dst + e0;
        const std::string where = " (graph " + std::to_string(b) + ")";
        for (int32_t e = 0; e < m; ++e) {
            if (src[e] < 0 || src[e] >= n || dst[e] < 0 || dst[e] >= n)
                return fail(PL_ERR_RANGE, "edge endpoint out of range" + where);
            if (src[e] == dst[e]) return fail(PL_ERR_SELF_LOOP, "self loop" + where);
        }
        fill_csr(n, m, dst, src, e0, &L.par_ptr[n0], &L.par_idx[e0]);
        fill_csr(n, m, src, dst, e0, &L.chi_ptr[n0], &L.chi_idx[e0]);
        for (int32_t v = 0; v < n; ++v)
            for (int64_t p = L.par_ptr[n0 + v] + 1; p < L.par_ptr[n0 + v + 1]; ++p)
                if (L.par_idx[p] == L.par_idx[p - 1])
                    return fail(PL_ERR_DUP_EDGE, "repeated edge" + where);
        if (!longest_path_levels(n, &L.par_ptr[n0], &L.chi_ptr[n0], &L.chi_idx[e0], e0,
                                 &L.td_level[n0]))
            return fail(PL_ERR_CYCLE, "graph has a cycle" + where);
        longest_path_levels(n, &L.chi_ptr[n0], &L.par_ptr[n0], &L.par_idx[e0], e0, &L.bu_level[n0]);
        const int32_t depth = 1 + *std::max_element(&L.td_level[n0], &L.td_level[n0] + n);
        L.depth[b] = depth;
        L.max_depth = std::max(L.max_depth, depth);
        L.lvl_off[b + 1] = L.lvl_off[b] + depth + 1;
    }

    L.td_lvl_ptr.resize(L.lvl_off[B]);
    L.bu_lvl_ptr.resize(L.lvl_off[B]);
    for (int32_t b = 0; b < B; ++b) {
        const int64_t n0 = L.node_off[b];
        bucket_by_level(n_nodes[b], L.depth[b], &L.td_level[n0], &L.td_order[n0],
                        &L.td_lvl_ptr[L.lvl_off[b]]);
        bucket_by_level(n_nodes[b], L.depth[b], &L.bu_level[n0], &L.bu_order[n0],
                        &L.bu_lvl_ptr[L.lvl_off[b]]);
    }
    L.n_templates = B;
    L.tmpl.resize(B);
    std::iota(L.tmpl.begin(), L.tmpl.end(), 0);
    L.tmpl_graph = L.tmpl;
    return PL_OK;
}

int replicate_layout(const HostLayout &one, int32_t R, HostLayout *out)
{
    if (one.B != 1) return fail(PL_ERR_SHAPE, "only a single graph can be replicated");
    if (R < 1) return fail(PL_ERR_SHAPE, "the number of copies must be at least 1");
    const int64_t n = one.n_tot, e = one.e_tot;
    if (n * R > INT32_MAX / 2 || e * R > INT32_MAX / 2)
        return fail(PL_ERR_SHAPE, "batch too large for 32-bit device indices");
    HostLayout &L = *out;
    L = HostLayout();
    L.B = R;
    L.n_tot = n * R;
    L.e_tot = e * R;
    L.max_depth = one.max_depth;
    L.depth.assign(R, one.depth[0]);
    L.node_off.resize(static_cast<size_t>(R) + 1);
    L.edge_off.resize(static_cast<size_t>(R) + 1);
    L.lvl_off.resize(static_cast<size_t>(R) + 1);
    for (int32_t r = 0; r <= R; ++r) {
        L.node_off[r] = n * r;
        L.edge_off[r] = e * r;
        L.lvl_off[r] = one.lvl_off[1] * r;
    }
    auto tile = [R](const auto &src, auto &dst) {      // the same values for every copy
        dst.reserve(src.size() * R);
        for (int32_t r = 0; r < R; ++r) dst.insert(dst.end(), src.begin(), src.end());
    };
    tile(one.par_idx, L.par_idx);
    tile(one.chi_idx, L.chi_idx);
    tile(one.td_level, L.td_level);
    tile(one.bu_level, L.bu_level);
    tile(one.td_order, L.td_order);
    tile(one.bu_order, L.bu_order);
    tile(one.td_lvl_ptr, L.td_lvl_ptr);
    tile(one.bu_lvl_ptr, L.bu_lvl_ptr);
    L.par_ptr.resize(L.n_tot + 1);                      // offsets into the batch-wide lists
    L.chi_ptr.resize(L.n_tot + 1);
    for (int32_t r = 0; r < R; ++r)
        for (int64_t v = 0; v <= n; ++v) {
            L.par_ptr[n * r + v] = one.par_ptr[v] + e * r;
            L.chi_ptr[n * r + v] = one.chi_ptr[v] + e * r;
        }
    L.n_templates = 1;
    L.tmpl.assign(R, 0);
    L.tmpl_graph.assign(1, 0);
    return PL_OK;
}

}  // namespace pl
