// Chunk plan of the matrix-core sweep kernel: constants and records shared by the host builder
// (plan.cpp) and the kernel (kernels_mfma.hip).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <vector>

namespace pl {

struct HostLayout;

// ---- gather plan of the matrix-core sweep kernel (plan.cpp)
constexpr int kChunkRows = 8;    // nodes per chunk: two MFMA row tiles of four nodes
constexpr int kFarCap = 16;      // far sources staged per chunk
constexpr int kRing = 2;         // chunks whose messages stay in the LDS table
constexpr int kMaxEnt = 20;      // neighbours per row held in the chunk record (6 bits each, 5 per word)
constexpr int kMsgSlots = kRing * kChunkRows + 2 * kFarCap;

struct SweepPlanHost {
    std::vector<int32_t> ck_off;   // [B+1] chunk range of each graph
    std::vector<int32_t> meta;     // [n_chunks][4]: global bucket position, rows, n_far,
                                   // most table entries of a row | (some row uses the overflow list) << 8
    std::vector<uint32_t> ent;     // [n_chunks][kChunkRows][4]: twenty 6-bit table slots, entry k in bits
                                   // 6 (k % 5) .. of word k / 5; unused entries = kMsgSlots, the table's
                                   // zero row.  Bit 30 of word 0 set: the row uses the overflow list
                                   // (word 1 = its offset in ovf, word 2 = its length)
    std::vector<int32_t> far;      // [n_chunks][kFarCap] global node ids staged for the chunk
    std::vector<int32_t> ovf;      // neighbour lists of rows that do not fit their record:
                                   // >= 0 global node id (>= 3 chunks back), < 0: -1 - table slot
    int64_t n_chunks = 0;
};

int build_sweep_plan(const HostLayout &L, int dir, SweepPlanHost *out);

struct SweepPlanView {
    const int32_t *ck_off;
    const int4 *meta;
    const uint4 *ent;
    const int32_t *far;
    const int32_t *ovf;
};

}  // namespace pl
