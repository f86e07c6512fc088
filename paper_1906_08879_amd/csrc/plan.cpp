// Host-side gather plan for the matrix-core sweep kernel.
//
// The sweep (Section 2.2 step 2) visits a graph level by level; a level is cut into chunks
// of at most kChunkRows nodes.  The kernel keeps the messages of the last kRing chunks in an
// LDS table and stages messages from older chunks ("far" sources) into the same table one
// chunk ahead.  This file turns the CSR into, per chunk: its position and row count, for
// every row the LDS table slots of its neighbours (unused entries name the table's zero row,
// slot kMsgSlots, so that a fixed number of entries can be summed without tests), and the
// list of far sources to stage.
#include <algorithm>
#include <cstdint>
#include <vector>

#include "internal.h"

namespace pl {

static_assert(kMsgSlots < 64 && kMaxEnt <= 20, "table slots are stored in six bits, twenty per record");

int build_sweep_plan(const HostLayout &L, int dir, SweepPlanHost *out)
{
    SweepPlanHost &P = *out;
    P = SweepPlanHost();
    const auto &ptr = dir ? L.chi_ptr : L.par_ptr;
    const auto &idx = dir ? L.chi_idx : L.par_idx;
    const auto &order = dir ? L.bu_order : L.td_order;
    const auto &lvl_ptr = dir ? L.bu_lvl_ptr : L.td_lvl_ptr;
    P.ck_off.assign(static_cast<size_t>(L.B) + 1, 0);
    std::vector<int32_t> node_chunk, node_row;
    for (int32_t b = 0; b < L.B; ++b) {
        const int64_t n0 = L.node_off[b];
        const int32_t n = static_cast<int32_t>(L.node_off[b + 1] - n0);
        const int32_t *lp = &lvl_ptr[L.lvl_off[b]];
        node_chunk.assign(n, 0);
        node_row.assign(n, 0);
        const int32_t first = static_cast<int32_t>(P.meta.size() / 4);
        // pass 1: cut levels into chunks
        for (int32_t level = 0; level < L.depth[b]; ++level) {
            for (int32_t p0 = lp[level]; p0 < lp[level + 1]; p0 += kChunkRows) {
                const int32_t rows = std::min(kChunkRows, lp[level + 1] - p0);
                const int32_t c = static_cast<int32_t>(P.meta.size() / 4) - first;
                for (int32_t r = 0; r < rows; ++r) {
                    node_chunk[order[n0 + p0 + r]] = c;
                    node_row[order[n0 + p0 + r]] = r;
                }
                P.meta.insert(P.meta.end(), {static_cast<int32_t>(n0) + p0, rows, 0, 0});
            }
        }
        const int32_t n_chunks = static_cast<int32_t>(P.meta.size() / 4) - first;
        P.ck_off[b + 1] = first + n_chunks;
        // every record starts as "no neighbours": all twenty entries the table's zero row
        {
            uint32_t empty = 0;
            for (int i = 0; i < 5; ++i) empty |= static_cast<uint32_t>(kMsgSlots) << (6 * i);
            P.ent.resize(static_cast<size_t>(first + n_chunks) * kChunkRows * 4, empty);
        }
        P.far.resize(static_cast<size_t>(first + n_chunks) * kFarCap, -1);
        // pass 2: neighbour slots
        for (int32_t c = 0; c < n_chunks; ++c) {
            int32_t *meta = &P.meta[static_cast<size_t>(first + c) * 4];
            int32_t *far = &P.far[static_cast<size_t>(first + c) * kFarCap];
            int32_t n_far = 0, max_ent = 0, has_ovf = 0;
            const int32_t p0 = meta[0] - static_cast<int32_t>(n0);
            for (int32_t r = 0; r < meta[1]; ++r) {
                uint32_t *ent = &P.ent[(static_cast<size_t>(first + c) * kChunkRows + r) * 4];
                const int32_t v = order[n0 + p0 + r];
                const int64_t e0 = ptr[n0 + v], e1 = ptr[n0 + v + 1];
                const int32_t deg = static_cast<int32_t>(e1 - e0);
                bool direct = deg > kMaxEnt;
                int32_t new_far = 0;
                if (!direct) {
                    for (int64_t e = e0; e < e1; ++e) {
                        const int32_t u = idx[e];
                        if (c - node_chunk[u] > kRing &&
                            std::find(far, far + n_far, static_cast<int32_t>(n0) + u) == far + n_far)
                            ++new_far;   // (a source repeated inside this row cannot occur: simple graph)
                    }
                    direct = n_far + new_far > kFarCap;
                }
                if (direct) {            // the row's list goes to the overflow array
                    const uint32_t off = static_cast<uint32_t>(P.ovf.size());
                    has_ovf = 1;
                    ent[0] |= 1u << 30;
                    ent[1] = off;
                    ent[2] = static_cast<uint32_t>(deg);
                    for (int64_t e = e0; e < e1; ++e) {
                        const int32_t u = idx[e];
                        if (c - node_chunk[u] <= kRing)
                            P.ovf.push_back(-1 - ((node_chunk[u] % kRing) * kChunkRows + node_row[u]));
                        else
                            P.ovf.push_back(static_cast<int32_t>(n0) + u);
                    }
                    continue;
                }
                max_ent = std::max(max_ent, deg);
                for (int64_t e = e0; e < e1; ++e) {
                    const int32_t u = idx[e];
                    int32_t slot;
                    if (c - node_chunk[u] <= kRing) {
                        slot = (node_chunk[u] % kRing) * kChunkRows + node_row[u];
                    } else {
                        const int32_t gu = static_cast<int32_t>(n0) + u;
                        int32_t f = static_cast<int32_t>(std::find(far, far + n_far, gu) - far);
                        if (f == n_far) far[n_far++] = gu;
                        slot = kRing * kChunkRows + (c % 2) * kFarCap + f;
                    }
                    const int k = static_cast<int>(e - e0);
                    ent[k / 5] = (ent[k / 5] & ~(63u << (6 * (k % 5)))) | (static_cast<uint32_t>(slot) << (6 * (k % 5)));
                }
            }
            meta[2] = n_far;
            meta[3] = max_ent | (has_ovf << 8);
        }
    }
    P.n_chunks = static_cast<int64_t>(P.meta.size() / 4);
    return PL_OK;
}

}  // namespace pl
