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
constexpr int kRing = 4;         // chunks whose messages stay in the LDS table
constexpr int kMaxNear = 5;      // table slots held in a row record (6 bits each)
constexpr int kMsgSlots = kRing * kChunkRows;   // table rows; row kMsgSlots is all zero
constexpr uint32_t kNoFar = 0xFFFFFFFFu;

// A row record is four 32-bit words; ids and positions are local to the graph, so that graphs of
// the same topology share one plan:
//   w0  five 6-bit table slots of "near" sources (computed at most kRing chunks ago), entry k in
//       bits 6k .., unused entries = kMsgSlots (the zero row); or, with bit 30 set, the row is
//       LISTED: bits 0..23 = number of its sources, all of which are in the list at w1
//   w1  the row's one "far" source (older than kRing chunks; read from HBM), kNoFar if none;
//       for a listed row the offset of its list in `ovf`
//   w2  bucket position of the chunk's first row
//   w3  bits 0..23 node id of the row (0xFFFFFF for the unused rows of a chunk),
//       bits 24..26 rows of the chunk - 1, bit 27 some row of the chunk is listed,
//       bit 28 some row of the chunk has a far source,
//       bits 29..30 near sources of the chunk's widest unlisted row: 0 = at most one, 1 = two, 2 = up to five
// A row is listed when it has more than kMaxNear near sources or more than one far source.
constexpr uint32_t kRecListed = 1u << 30;
constexpr int kRecRowsShift = 24, kRecGeneralBit = 27, kRecFarBit = 28, kRecNearShift = 29;
constexpr uint32_t kRecNoNode = 0xFFFFFFu;

struct SweepPlanHost {
    std::vector<int32_t> ck_off;   // [n_templates + 1] chunk range of each distinct graph
    std::vector<uint32_t> rec;     // [n_chunks][kChunkRows][4] row records
    std::vector<int32_t> ovf;      // source lists of listed rows: >= 0 node id (far), < 0: -1 - table slot
    int64_t n_chunks = 0;
};

int build_sweep_plan(const HostLayout &L, int dir, SweepPlanHost *out);

struct SweepPlanView {
    const int32_t *ck_off;
    const uint4 *rec;
    const int32_t *ovf;
};

}  // namespace pl
