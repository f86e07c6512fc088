// Host-side gather plan for the matrix-core sweep kernel.
//
// The sweep (Section 2.2 step 2) visits a graph level by level; a level is cut into chunks
// of at most kChunkRows nodes.  The kernel keeps the messages of the last kRing chunks in an
// LDS table ("near" sources) and reads older messages ("far" sources) back from HBM, two
// chunks ahead of their use.  This file turns the CSR into one 16-byte record per chunk row:
// the table slots of its near sources, its far source, where the chunk starts in the bucket
// order, and the node id; rows with more sources than a record holds get a list.  Everything
// is local to the graph, and graphs of the same topology (rollouts of one graph) share a plan.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "internal.h"

namespace pl {

static_assert(kMsgSlots < 64 && kMaxNear <= 5, "table slots are stored in six bits, five per word");

int build_sweep_plan(const HostLayout &L, int dir, SweepPlanHost *out)
{
    SweepPlanHost &P = *out;
    P = SweepPlanHost();
    const auto &ptr = dir ? L.chi_ptr : L.par_ptr;
    const auto &idx = dir ? L.chi_idx : L.par_idx;
    const auto &order = dir ? L.bu_order : L.td_order;
    const auto &lvl_ptr = dir ? L.bu_lvl_ptr : L.td_lvl_ptr;
    P.ck_off.assign(static_cast<size_t>(L.n_templates) + 1, 0);
    std::vector<int32_t> node_chunk, node_row;
    uint32_t empty_slots = 0;
    for (int i = 0; i < kMaxNear; ++i) empty_slots |= static_cast<uint32_t>(kMsgSlots) << (6 * i);
    for (int32_t t = 0; t < L.n_templates; ++t) {
        const int32_t b = L.tmpl_graph[t];
        const int64_t n0 = L.node_off[b];
        const int32_t n = static_cast<int32_t>(L.node_off[b + 1] - n0);
        if (n > static_cast<int32_t>(kRecNoNode)) return fail(PL_ERR_SHAPE, "a graph has more than 2^24 - 1 nodes");
        const int32_t *lp = &lvl_ptr[L.lvl_off[b]];
        node_chunk.assign(n, 0);
        node_row.assign(n, 0);
        const size_t first = P.rec.size() / (kChunkRows * 4);
        // pass 1: cut levels into chunks
        std::vector<int32_t> start, rows_of;
        for (int32_t level = 0; level < L.depth[b]; ++level)
            for (int32_t p0 = lp[level]; p0 < lp[level + 1]; p0 += kChunkRows) {
                const int32_t rows = std::min(kChunkRows, lp[level + 1] - p0);
                const int32_t c = static_cast<int32_t>(start.size());
                for (int32_t r = 0; r < rows; ++r) {
                    node_chunk[order[n0 + p0 + r]] = c;
                    node_row[order[n0 + p0 + r]] = r;
                }
                start.push_back(p0);
                rows_of.push_back(rows);
            }
        const int32_t n_chunks = static_cast<int32_t>(start.size());
        P.ck_off[t + 1] = static_cast<int32_t>(first) + n_chunks;
        P.rec.resize((first + n_chunks) * kChunkRows * 4, 0);
        // pass 2: one record per row
        for (int32_t c = 0; c < n_chunks; ++c) {
            uint32_t *rec = &P.rec[(first + c) * kChunkRows * 4];
            int32_t max_near = 0;
            bool any_far = false, any_listed = false;
            for (int32_t r = 0; r < kChunkRows; ++r) {
                uint32_t *w = rec + 4 * r;
                w[0] = empty_slots;
                w[1] = kNoFar;
                w[2] = static_cast<uint32_t>(start[c]);
                w[3] = kRecNoNode;
                if (r >= rows_of[c]) continue;
                const int32_t v = order[n0 + start[c] + r];
                w[3] = static_cast<uint32_t>(v);
                const int64_t e0 = ptr[n0 + v], e1 = ptr[n0 + v + 1];
                int32_t near = 0, far = 0;
                for (int64_t e = e0; e < e1; ++e) (c - node_chunk[idx[e]] <= kRing ? near : far) += 1;
                if (near > kMaxNear || far > 1) {     // all sources of the row go to a list
                    any_listed = true;
                    w[0] = kRecListed | static_cast<uint32_t>(e1 - e0);
                    w[1] = static_cast<uint32_t>(P.ovf.size());
                    for (int64_t e = e0; e < e1; ++e) {
                        const int32_t u = idx[e];
                        if (c - node_chunk[u] <= kRing)
                            P.ovf.push_back(-1 - ((node_chunk[u] % kRing) * kChunkRows + node_row[u]));
                        else
                            P.ovf.push_back(u);
                    }
                    continue;
                }
                max_near = std::max(max_near, near);
                int k = 0;
                for (int64_t e = e0; e < e1; ++e) {
                    const int32_t u = idx[e];
                    if (c - node_chunk[u] <= kRing) {
                        const uint32_t slot = static_cast<uint32_t>((node_chunk[u] % kRing) * kChunkRows + node_row[u]);
                        w[0] = (w[0] & ~(63u << (6 * k))) | (slot << (6 * k));
                        ++k;
                    } else {
                        w[1] = static_cast<uint32_t>(u);
                        any_far = true;
                    }
                }
            }
            const uint32_t chunk_bits = (static_cast<uint32_t>(rows_of[c] - 1) << kRecRowsShift) |
                                        (any_listed ? 1u << kRecGeneralBit : 0u) | (any_far ? 1u << kRecFarBit : 0u) |
                                        (static_cast<uint32_t>(max_near <= 1 ? 0 : (max_near == 2 ? 1 : 2)) << kRecNearShift);
            for (int32_t r = 0; r < kChunkRows; ++r) rec[4 * r + 3] |= chunk_bits;
        }
    }
    P.n_chunks = static_cast<int64_t>(P.rec.size() / (kChunkRows * 4));
    if (P.ovf.size() >= (1u << 30)) return fail(PL_ERR_SHAPE, "source lists of the sweep plan too long");
    return PL_OK;
}

}  // namespace pl
