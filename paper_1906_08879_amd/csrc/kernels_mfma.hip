// Matrix-core sweep kernel for gfx950: the message passing of Section 2.2 step 2,
//   a_v = sum_{u in xi(v)} m_u,   s_v <- s_v + g(a_v),   m_v = f(s_v),
// for H in {32, 64, 128} and one or two layers per network.
//
// One workgroup (one wave per 16 or 32 output columns, at most four waves) per (graph, direction)
// walks the graph's levels in chunks of at most 8 nodes.  Design points, all specific to
// CDNA4:
//   * v_mfma_f32_16x16x32_bf16 with the node activations as the A operand and the WEIGHTS as
//     the B operand.  The fp32 activation of a node is split exactly into three bf16 values
//     (hi, mid, lo) by truncation; the three parts are three ROWS of A (a fourth row is
//     zero), so a 16-row tile holds four nodes and the three partial products of a node land
//     in one lane's accumulator registers, where they are added: fp32 accuracy from the bf16
//     matrix cores without any cross-lane traffic.
//   * The weight fragments of all layers of one direction live in registers for the whole
//     kernel (bf16 weights: 128 VGPRs per wave at H = 128); only activations move through LDS.
//     A lane that owns two output columns owns NEIGHBOURS (a wave's two column tiles hold the
//     even and the odd columns of its 32): it writes them as ONE 32-bit word per bf16 part (three
//     conflict-free word stores per lane and row instead of six half-word stores), and reads or
//     writes them in HBM and in the message table with one 8-byte access.
//   * A wave owns its output columns from end to end: it writes its columns of a message into
//     an LDS table that holds the last kRing chunks ("near" sources), reads its columns of
//     older messages ("far" sources) back from HBM straight into the registers that sum them,
//     two chunks ahead of their use, and sums its columns for the next chunk, in the MFMA result
//     layout (lane = node of the tile, column).  The table therefore needs no barrier; only the
//     A rows of the next layer cross waves: one LDS barrier per layer, four per chunk.
//   * Messages are ReLU outputs, so their sign bit carries the reachability flag of Section 2.2
//     step 3 (the node is v* or was computed from v*), in the table and in HBM alike: sums take
//     |x| and OR the signs.  A row record names a fixed number of table slots (unused ones the
//     table's zero row) and one far source (or a row of zeros), so the common gather is
//     branch-free; rows with more sources walk a list.
//   * On the first sweep the same lane computes its columns of x_v = relu(W_in^T phi_v + b)
//     (step 1) from the node's 16-byte feature record: x never exists in HBM.
//   * Everything a chunk needs from HBM (row records three chunks ahead, feature records one,
//     far messages two) is loaded by plain vector loads behind the matrix instructions of an
//     earlier chunk; barriers order LDS traffic only, so those loads stay in flight across them.
//     A far message was stored by this same wave at least kRing + 1 chunks before it is used and
//     at least kRing - 1 chunks before it is loaded; in between the wave has waited for loads that
//     it issued after that store, so the store has retired.
//   * The kernel runs a dependent chain (about a thousand chunks of four layers per graph),
//     so it is bound by LDS round trips, MFMA latency and barriers, not by HBM bandwidth.
#include <type_traits>

#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int CH = kChunkRows, RING = kRing;
constexpr int kTileNodes = 4;                 // nodes per 16-row MFMA tile (hi, mid, lo, zero rows)
constexpr int NT = CH / kTileNodes;           // row tiles per chunk

// Workgroup barrier that orders LDS traffic only: global loads and stores stay outstanding.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ float trunc_bf16(float x)
{
    return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u);
}

// {high half of a, high half of b} as one word, a in the low half
__device__ __forceinline__ uint32_t pack_hi16(float a, float b)
{
    return __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
}

struct SweepParams {
    GraphView gv;
    const uint4 *wfrag;     // packed weight fragments, see pack_sweep_weights()
    const float *bias;      // [2 dir][2L layers][H]
    float *emb;             // [n_tot, 2H]   output s_v in node order ([td ; bu])
    float *xb;              // [2, n_tot, H] residual input in bucket order, per direction
    float *msg;             // [2, n_tot, H]
    uint8_t *reach;         // [2, n_tot]
    const int32_t *cur_node;
    // first sweep: the input x_v = relu(W_in^T phi_v + b_in) (Section 2.2 step 1) is computed
    // here from the node's raw features, 16 bytes per node
    const float4 *featb;    // [n_tot] {run time, output size, is-visited, bits(device | is-current << 16)}, node order
    const float *proj;      // [(F + 1), H]: rows of W_in, then b_in; NULL when the input comes from xb
    int D;
    // ReLU gates of every node's layers, one byte per (sweep direction, node, column), node order:
    // bit 0 m_v > 0 (gates the gathered sum of the reverse pass), bit 1 output of f's layer 0 > 0
    // (L = 2), bit 2 output of g's last layer > 0, bit 3 output of g's layer 0 > 0 (L = 2).
    // Written by a sweep that keeps activations (TR), read by the reverse pass (BW); row 2 n_tot
    // takes the stores of a chunk's unused rows.
    uint8_t *mask4;         // [2 n_tot + 1, H]
    float *delta;           // per sweep direction: [2L][n_tot, H] (f's layers, then g's), then H
                            // floats that take the stores of a chunk's unused rows
    size_t delta_stride;    // floats between the two directions' blocks
};

constexpr int sweep_waves(int H) { return H / 16 > 4 ? 4 : H / 16; }

// FF: first sweep, the input x_v is computed from the raw-feature records; otherwise it is
// read from xb.  WX: another sweep follows, s_v is also written to xb.
// BW: the reverse pass of a sweep, which has the same shape.  With the chunks of the OTHER
// direction (a node's gradient needs those of the nodes that gathered its message, and those
// come earlier in the other direction's level order) and the transposed weights in the order
// f then g, a chunk is: gathered sum of da over the consumers, gated by m_v > 0; back through
// the layers of f; + the outside gradient of s_v (read where the forward pass reads x_v) =
// ds_v, written where the forward pass writes s_v; gated, back through the layers of g; the
// result da_v goes where the forward pass puts the message.  ReLU and bias are replaced by the
// stored gates, table entries and stored values are signed (no reachability flag), and every
// gated layer input is also written to HBM as the layer's delta for the weight gradients.
// TR: a forward sweep that also keeps what the reverse pass needs of every node: the gathered
// sum a_v and the output of every layer but the last (the last is the message, stored anyway),
// 2L arrays [n_tot, H] per direction in `delta` (slot 0: a_v, slots 1 .. L: g's layers, slots
// L + 1 .. 2L - 1: f's layers but the last).
template <int H, int WS, int L, bool FF, bool WX, bool BW = false, bool TR = false>
__global__ __launch_bounds__(64 * sweep_waves(H), 2) void k_sweep_mfma(SweepParams P)
{
    static_assert(!BW || (!FF && !WX), "the reverse pass reads its input from xb and writes no xb");
    static_assert(!TR || (FF && !WX && !BW), "activations are kept for a single forward sweep");
    constexpr int NW = sweep_waves(H);         // waves; wave w owns output columns [w WC, (w + 1) WC)
    constexpr int kThreads = 64 * NW;
    constexpr int NTL = H / 16, KS = H / 32;
    constexpr int TPW = NTL / NW;              // output column tiles per wave
    constexpr int WC = 16 * TPW;               // columns owned by a wave
    constexpr int NL = 2 * L;                  // layers per chunk: g then f
    // bf16 row stride of the activation buffers: H / 2 + 8 words.  Measured with
    // SQ_LDS_BANK_CONFLICT on this chip: the ds_read_b128 of A rows (lane = row, 16-byte piece)
    // then runs at its full rate of four cycles (a stride of H / 2 + 4 words takes eight), while
    // the word stores of a tile's four nodes take four cycles instead of two; no skew of the rows
    // tried (multiples of four words on rows 4..7 and 8..15) is free of conflicts for both.
    constexpr int LDA = H + 16;
    constexpr int kActTile = 16 * LDA;         // one 16-row tile
    constexpr int LDM = H + 16;                // float row stride of the message table (16 mod 64:
                                               // four consecutive rows fall on disjoint banks)
    constexpr int kZeroSlot = kMsgSlots;
    static_assert(NTL % NW == 0, "column tiles must divide over the waves");
    static_assert(TPW == 1 || TPW == 2, "a lane owns one or two output columns");
    constexpr bool kReadFirst = TPW == 1;
#ifndef PL_SINK_STORES
#define PL_SINK_STORES 0
#endif
    constexpr bool kSinkStores = PL_SINK_STORES;
#ifndef PL_UNCOND_T1
#define PL_UNCOND_T1 0
#endif
    // What a later chunk's second row tile needs is loaded whether or not that chunk has one
    // (its records then name the all-zero rows): no branch splits the code of a layer.  The
    // reverse pass, which loads four values per row and column tile, keeps the test.
    constexpr bool kLoadTile1Always = PL_UNCOND_T1;
#ifndef PL_SPLIT_KINDS
#define PL_SPLIT_KINDS (!BW)
#endif
    constexpr bool kSplitKinds = PL_SPLIT_KINDS;
    // A forward sweep writes what the next layer waits for to LDS before it stores to HBM; the
    // variants that keep activations or feed another sweep have no registers to hold the values
    // meanwhile.
    constexpr bool kLdsFirst = !BW && !TR && !WX;

    // Message table: H floats per row.  Messages are ReLU outputs, so their sign bit is free:
    // it carries the reachability flag of the row's node (set if the node is v* or has v* among
    // the nodes it was computed from); sums take |x|.  A wave reads and writes only its own
    // columns, so the table needs no barrier.  The last row stays zero.
    __shared__ __attribute__((aligned(16))) float msgtab[(kMsgSlots + 1) * LDM];
    __shared__ __attribute__((aligned(16))) __bf16 actbuf[2][NT * kActTile];
    // element (row r of the chunk's 16 NT rows, column k) of buffer `buf`
    auto act_at = [&](int buf, int r, int k) __attribute__((always_inline)) {
        return &actbuf[buf][r * LDA + k];
    };
    __shared__ float proj_dev[(kMaxD + 1) * H];   // one-hot device rows of W_in, then a zero row
    __shared__ float proj_row[TR ? 5 * H : 1];    // (TR) the other rows of W_in and its bias
    __shared__ float bias_row[(TR || (FF && WX)) ? 2 * L * H : 1];   // the layers' biases, for the variants short of registers

    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;    // MFMA result: column col, node kg of a tile
    const int wc0 = wave * WC;
    // Output column of this lane in the wave's column tile t.  Where a wave owns two tiles they
    // interleave (tile 0 the even, tile 1 the odd columns of the wave's 32), so that a lane's two
    // columns are neighbours: one 8-byte access per lane wherever a row is read or written.
    auto mcol = [&](int t) __attribute__((always_inline)) { return wc0 + (TPW == 2 ? 2 * col + t : col); };
    // this lane's columns of a row of floats that starts at element `at`
    auto load_cols = [&](const float *base, uint32_t at, float (&v)[TPW]) __attribute__((always_inline)) {
        if constexpr (TPW == 2) {
            const float2 x = *reinterpret_cast<const float2 *>(base + static_cast<uint32_t>(at + mcol(0)));
            v[0] = x.x;
            v[1] = x.y;
        } else {
            v[0] = base[static_cast<uint32_t>(at + mcol(0))];
        }
    };
    // the same for rows of gate bytes
    auto load_gates = [&](const uint8_t *base, uint32_t at, int (&v)[TPW]) __attribute__((always_inline)) {
        if constexpr (TPW == 2) {
            const int x = *reinterpret_cast<const uint16_t *>(base + static_cast<uint32_t>(at + mcol(0)));
            v[0] = x & 0xFF;
            v[1] = x >> 8;
        } else {
            v[0] = base[static_cast<uint32_t>(at + mcol(0))];
        }
    };
    auto store_gates = [&](uint8_t *base, uint32_t at, const int (&v)[TPW]) __attribute__((always_inline)) {
        if constexpr (TPW == 2)
            *reinterpret_cast<uint16_t *>(base + static_cast<uint32_t>(at + mcol(0))) = static_cast<uint16_t>(v[0] | (v[1] << 8));
        else
            base[static_cast<uint32_t>(at + mcol(0))] = static_cast<uint8_t>(v[0]);
    };
    auto store_cols = [&](float *base, uint32_t at, const float (&v)[TPW]) __attribute__((always_inline)) {
        if constexpr (TPW == 2)
            *reinterpret_cast<float2 *>(base + static_cast<uint32_t>(at + mcol(0))) = float2{v[0], v[1]};
        else
            base[static_cast<uint32_t>(at + mcol(0))] = v[0];
    };

    const GraphView &gv = P.gv;
    const SweepPlanView plan = gv.plan[dir];
    float *msg = P.msg + static_cast<size_t>(dir) * gv.n_tot * H;
    float *xb = P.xb + static_cast<size_t>(dir) * gv.n_tot * H;
    uint8_t *reach = P.reach + static_cast<size_t>(dir) * gv.n_tot;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = P.cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const int tm = gv.tmpl[b];
    const int c_begin = plan.ck_off[tm], c_end = plan.ck_off[tm + 1];
    if (c_begin >= c_end) return;
    // one row past both directions' messages is never written and reads as zero: the address of
    // the loads of rows without a far source, relative to this direction's base.  The row after
    // it (and the byte past both directions' bits, and row n_tot of emb) take the stores of a
    // chunk's unused rows: every lane stores on every chunk, so the number of stores in flight
    // behind a load is known when the kernel is compiled and a wait for that load does not wait
    // for the stores.
    const int spare_row = (2 - dir) * gv.n_tot;
    const int sink_row = spare_row + 1;

    // ---- weights of this direction into registers (B operand: lane holds column 16 nt + col)
    // The variants that keep activations, or compute the projection and feed another sweep, have
    // no registers for the biases: they read them from LDS.
    constexpr bool kBiasLds = TR || (FF && WX);
    bf16x8 W[NL][TPW][KS][WS];
    float bias[NL][TPW];
    if constexpr (kBiasLds)
        for (int i = tid; i < NL * H; i += kThreads) bias_row[i] = P.bias[static_cast<size_t>(dir) * NL * H + i];
#pragma unroll
    for (int n = 0; n < NL; ++n)
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int nt = wave * TPW + t;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int ws = 0; ws < WS; ++ws) {
                    const size_t at =
                        ((((static_cast<size_t>(dir) * NL + n) * NTL + nt) * KS + ks) * WS + ws) * 64 + lane;
                    const uint4 raw = P.wfrag[at];
                    W[n][t][ks][ws] = *reinterpret_cast<const bf16x8 *>(&raw);
                }
            if constexpr (!kBiasLds) bias[n][t] = P.bias[(static_cast<size_t>(dir) * NL + n) * H + mcol(t)];
        }

    // ---- input projection (Section 2.2 step 1), one output column per lane and tile:
    // x = relu(b + time w0 + size w1 + w[2 + device] + is_current w[2 + D] + visited w[3 + D])
    const int D = P.D;
    // The five rows of W_in that do not depend on the device stay in registers, except in the
    // variant that keeps activations, which has no registers to spare: it reads them from LDS.
    constexpr bool kProjLds = TR;
    float pw_time[TPW], pw_size[TPW], pw_cur[TPW], pw_vis[TPW], pw_b[TPW];
    if constexpr (FF) {
        if constexpr (kProjLds) {
            for (int i = tid; i < H; i += kThreads) {
                proj_row[0 * H + i] = P.proj[i];
                proj_row[1 * H + i] = P.proj[H + i];
                proj_row[2 * H + i] = P.proj[(2 + D) * H + i];
                proj_row[3 * H + i] = P.proj[(3 + D) * H + i];
                proj_row[4 * H + i] = P.proj[(4 + D) * H + i];
            }
        } else {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int m = mcol(t);
                pw_time[t] = P.proj[m];
                pw_size[t] = P.proj[H + m];
                pw_cur[t] = P.proj[(2 + D) * H + m];
                pw_vis[t] = P.proj[(3 + D) * H + m];
                pw_b[t] = P.proj[(4 + D) * H + m];
            }
        }
        for (int i = tid; i < (kMaxD + 1) * H; i += kThreads)
            proj_dev[i] = (i < D * H) ? P.proj[2 * H + i] : 0.0f;
    }
    const float4 *featb = P.featb;   // one 16-byte record per node, node order
    // the device's row of W_in comes from LDS: read early (device_term), used late (project)
    auto device_term = [&](const f32x4 ft, int t) __attribute__((always_inline)) {
        const int dev = __float_as_int(ft[3]) & 0xFFFF;
        return proj_dev[(dev < D ? dev : D) * H + mcol(t)];
    };
    auto project = [&](const f32x4 ft, float dev_term, int t) __attribute__((always_inline)) {
        const int bits = __float_as_int(ft[3]);
        const int m = mcol(t);
        const float w_time = kProjLds ? proj_row[0 * H + m] : pw_time[t], w_size = kProjLds ? proj_row[1 * H + m] : pw_size[t];
        const float w_cur = kProjLds ? proj_row[2 * H + m] : pw_cur[t], w_vis = kProjLds ? proj_row[3 * H + m] : pw_vis[t];
        float o = kProjLds ? proj_row[4 * H + m] : pw_b[t];
        o = fmaf(ft[0], w_time, o);
        o = fmaf(ft[1], w_size, o);
        o += dev_term;
        o += (bits >> 16) ? w_cur : 0.0f;
        return fmaxf(fmaf(ft[2], w_vis, o), 0.0f);
    };
    for (int i = tid; i < (kMsgSlots + 1) * LDM; i += kThreads) msgtab[i] = 0.0f;
    for (int i = tid; i < 2 * NT * kActTile; i += kThreads) (&actbuf[0][0])[i] = static_cast<__bf16>(0.0f);

    // Writes this lane's values of node row r, split exactly into three bf16 parts, as rows
    // 4 r .. 4 r + 2 of an A operand.  Two columns per lane travel as one word per part: word
    // 16 wave + col of a row holds columns wc0 + 2 col (low half) and wc0 + 2 col + 1 (high half),
    // so the rows are in the natural order of the contraction index.
    auto put_rows = [&](int buf, int r, const float (&y)[TPW]) __attribute__((always_inline)) {
        float rr[TPW], ll[TPW];
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            rr[t] = y[t] - trunc_bf16(y[t]);
            ll[t] = rr[t] - trunc_bf16(rr[t]);
        }
        if constexpr (TPW == 2) {
            uint32_t *dst = reinterpret_cast<uint32_t *>(act_at(buf, 4 * r, 0)) + 16 * wave + col;
            dst[0] = pack_hi16(y[0], y[1]);
            dst[LDA / 2] = pack_hi16(rr[0], rr[1]);
            dst[LDA] = pack_hi16(ll[0], ll[1]);
        } else {
            unsigned short *dst = reinterpret_cast<unsigned short *>(act_at(buf, 4 * r, wc0 + col));
            dst[0] = static_cast<unsigned short>(__float_as_uint(y[0]) >> 16);
            dst[LDA] = static_cast<unsigned short>(__float_as_uint(rr[0]) >> 16);
            dst[2 * LDA] = static_cast<unsigned short>(__float_as_uint(ll[0]) >> 16);
        }
    };

    // ---- gather of a chunk: a_v = sum of neighbour messages, for rows kg and kg + 4 and this
    // wave's columns: K table slots of the row's record (unused entries name the zero row) and
    // the row's far message, which is already in registers (zeros if the row has none); written
    // as A rows of the first layer.  Reverse pass: the sum is gated by bit 0 of the row's mask
    // and kept in gs (it is the delta of f's last layer, stored when the chunk is processed).
    // A sweep that keeps activations (TR) stores the sum right here (w3 = word 3 of the row's
    // record: its node id), slot 0 of the kept arrays.
    auto finish_row = [&](int ct, float (&s)[TPW], uint32_t signs, int (&bit)[NT], const int (&mk)[NT][TPW],
                          float (&gs)[NT][TPW], uint32_t w3) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            if constexpr (BW) {
                s[t] = (mk[ct][t] & 1) ? s[t] : 0.0f;
                gs[ct][t] = s[t];
            }
        }
        if constexpr (TR) {
            const uint32_t id = w3 & kRecNoNode;
            float *kept = P.delta + static_cast<size_t>(dir) * P.delta_stride;
            store_cols(kept, id == kRecNoNode ? static_cast<uint32_t>(2 * L * gv.n_tot * H)
                                              : static_cast<uint32_t>((n0 + static_cast<int>(id)) * H), s);
        }
        put_rows(0, 4 * ct + kg, s);
        bit[ct] = static_cast<int>(signs >> 31);
    };
    auto sum_slots = [&](auto kc, uint32_t slots, const float (&far)[TPW], float (&s)[TPW], uint32_t &signs) __attribute__((always_inline)) {
        constexpr int K = decltype(kc)::value;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            s[t] = BW ? far[t] : fabsf(far[t]);
            if (!BW && t == 0) signs |= __float_as_uint(far[t]);
        }
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int slot = static_cast<int>((slots >> (6 * k)) & 63u);
            const float *row = msgtab + slot * LDM;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const float x = row[mcol(t)];
                s[t] += BW ? x : fabsf(x);
                if (!BW && t == 0) signs |= __float_as_uint(x);
            }
        }
    };
    auto gather_fixed = [&](auto kc, int ntile_x, const u32x4 (&rec)[NT], const float (&far)[NT][TPW], int (&bit)[NT],
                            const int (&mk)[NT][TPW], float (&gs)[NT][TPW]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            bit[ct] = 0;
            if (ct >= ntile_x) continue;
            float s[TPW];
            uint32_t signs = 0;
            sum_slots(kc, rec[ct][0], far[ct], s, signs);
            finish_row(ct, s, signs, bit, mk, gs, rec[ct][3]);
        }
    };
    // The same for a chunk in which some row has more sources than its record holds: that row
    // sums a list of table slots (near sources) and node ids (far sources, read from HBM here).
    auto gather_general = [&](int ntile_x, const u32x4 (&rec)[NT], const float (&far)[NT][TPW], int (&bit)[NT],
                              const int (&mk)[NT][TPW], float (&gs)[NT][TPW]) __attribute__((always_inline)) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            bit[ct] = 0;
            if (ct >= ntile_x) continue;
            float s[TPW];
            uint32_t signs = 0;
            if ((rec[ct][0] & kRecListed) == 0) {
                sum_slots(std::integral_constant<int, kMaxNear>{}, rec[ct][0], far[ct], s, signs);
            } else {
#pragma unroll
                for (int t = 0; t < TPW; ++t) s[t] = 0.0f;
                const int d0 = static_cast<int>(rec[ct][1]);
                const int d1 = d0 + static_cast<int>(rec[ct][0] & 0xFFFFFFu);
                // An entry is a table slot or a node id; the other source of the pair is the
                // table's zero row or the spare (all-zero, never written) row of msg, so both are
                // always read and added, in list order.
                if constexpr (TPW == 1) {
                    // The list is walked in passes of PB entries, three passes per step.  The
                    // sixteen lanes of the row's group first load the step's entries (one load
                    // each per pass, all in flight together) and hand them round with lane
                    // shuffles; then a pass issues all its loads before the first use.
                    constexpr int PB = 16;
                    for (int p0 = d0; p0 < d1; p0 += 3 * PB) {
                        int idv[3];
#pragma unroll
                        for (int q = 0; q < 3; ++q) {
                            const int at = p0 + q * PB + (col % PB);
                            idv[q] = (at < d1) ? plan.ovf[at] : -1 - kZeroSlot;
                        }
#pragma unroll
                        for (int q = 0; q < 3; ++q) {
                            if (p0 + q * PB >= d1) break;
                            float xl[PB], xg[PB];
#pragma unroll
                            for (int k = 0; k < PB; ++k) {
                                const int u = __shfl(idv[q], (lane & 48) + k);
                                const float *row = msgtab + (u < 0 ? -1 - u : kZeroSlot) * LDM;
                                const int v = u >= 0 ? n0 + u : spare_row;
                                xl[k] = row[wc0 + col];
                                xg[k] = msg[static_cast<uint32_t>(v * H + wc0 + col)];
                            }
#pragma unroll
                            for (int k = 0; k < PB; ++k) {
                                s[0] += BW ? xl[k] + xg[k] : fabsf(xl[k]) + fabsf(xg[k]);
                                if (!BW) signs |= __float_as_uint(xl[k]) | __float_as_uint(xg[k]);
                            }
                        }
                    }
                } else {
                    // two column tiles per wave leave no registers for that: four entries at a time
                    for (int p = d0; p < d1; p += 4) {
                        int u[4];
#pragma unroll
                        for (int k = 0; k < 4; ++k) u[k] = p + k < d1 ? plan.ovf[p + k] : -1 - kZeroSlot;
                        float xl[4][TPW], xg[4][TPW];
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const float *row = msgtab + (u[k] < 0 ? -1 - u[k] : kZeroSlot) * LDM;
                            const int v = u[k] >= 0 ? n0 + u[k] : spare_row;
#pragma unroll
                            for (int t = 0; t < TPW; ++t) {
                                xl[k][t] = row[mcol(t)];
                                xg[k][t] = msg[static_cast<uint32_t>(v * H + mcol(t))];
                            }
                        }
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t)
                                s[t] += BW ? xl[k][t] + xg[k][t] : fabsf(xl[k][t]) + fabsf(xg[k][t]);
                            if (!BW) signs |= __float_as_uint(xl[k][0]) | __float_as_uint(xg[k][0]);
                        }
                    }
                }
            }
            finish_row(ct, s, signs, bit, mk, gs, rec[ct][3]);
        }
    };
    // info = word 3 of a record of the chunk (its chunk-wide bits)
    auto gather = [&](uint32_t info, const u32x4 (&rec)[NT], const float (&far)[NT][TPW], int (&bit)[NT],
                      const int (&mk)[NT][TPW], float (&gs)[NT][TPW]) __attribute__((always_inline)) {
        const int ntile_x = (static_cast<int>((info >> kRecRowsShift) & 7u) + kTileNodes) / kTileNodes;
        const int cls = static_cast<int>((info >> kRecNearShift) & 3u);
        if ((info >> kRecGeneralBit) & 1u)
            gather_general(ntile_x, rec, far, bit, mk, gs);
        else if (cls == 0)
            gather_fixed(std::integral_constant<int, 1>{}, ntile_x, rec, far, bit, mk, gs);
        else if (cls == 1)
            gather_fixed(std::integral_constant<int, 2>{}, ntile_x, rec, far, bit, mk, gs);
        else
            gather_fixed(std::integral_constant<int, kMaxNear>{}, ntile_x, rec, far, bit, mk, gs);
    };
    auto rows_of = [](uint32_t info) __attribute__((always_inline)) { return static_cast<int>((info >> kRecRowsShift) & 7u) + 1; };

    // ---- software pipeline state.  A lane works on rows kg (tile 0) and kg + 4 (tile 1) of a
    // chunk.  Everything that is loaded for a later chunk lives in a pair of register sets that
    // swap roles from chunk to chunk (the chunk loop is unrolled by two): a register that a load is still filling is never copied, so no wait falls earlier
    // than the first real use of the data.
    //   rcA            records of chunk c + 1 (arrived)
    //   rcX0 / rcX1    records of chunk c + 2 (loaded during chunk c - 1) / target of the records
    //                  of chunk c + 3
    //   ftp0 / ftp1    raw-feature records of chunk c (FF) / target for chunk c + 1
    //   xs, mks        the same for residual inputs and gate bytes (!FF / BW)
    //   farp0 / farp1  far messages of chunk c + 1 / target for chunk c + 2
    // Of chunk c itself only the node ids, the row count and the bucket position are kept.
    auto clampc = [&](int c) __attribute__((always_inline)) { return c < c_end ? c : c_end - 1; };
    auto load_rec = [&](int c, int ct) __attribute__((always_inline)) {
        return *reinterpret_cast<const u32x4 *>(plan.rec + static_cast<size_t>(clampc(c)) * CH + 4 * ct + kg);
    };
    u32x4 rcA[NT], rcX0[NT], rcX1[NT];
    int vg0[NT];             // global node ids of the rows of chunk c (any valid id for unused rows)
    int rows0, p0;           // rows and first bucket position (within the graph) of chunk c
    f32x4 ftp0[NT], ftp1[NT];
    float x0[NT][TPW];       // (FF) residual inputs x_v of chunk c, computed from its feature records
    float xs0[NT][TPW], xs1[NT][TPW];
    int mks0[NT][TPW], mks1[NT][TPW];
    int bit0[NT];            // reachability bits of the rows of chunk c
    float farp0[NT][TPW], farp1[NT][TPW];
    float gs0[NT][TPW];      // (BW) gated gathered sums of chunk c: the delta of f's last layer
    // the reverse pass works on sweep direction 1 - dir: it reads the outside gradient of a node's
    // state from emb (where it later writes the state's full gradient) and the node's gate bytes,
    // both by node id; a later forward sweep reads its input from xb in bucket order
    const uint8_t *gates_in = BW ? P.mask4 + static_cast<size_t>(1 - dir) * gv.n_tot * H : nullptr;
    uint8_t *gates_out = TR ? P.mask4 + static_cast<size_t>(dir) * gv.n_tot * H : nullptr;
    const float *xin = xb + static_cast<size_t>(n0) * H;
    auto node_of = [&](const u32x4 &rec) __attribute__((always_inline)) {
        const uint32_t id = rec[3] & kRecNoNode;
        return n0 + static_cast<int>(id == kRecNoNode ? 0u : id);
    };
    float *dlt = BW ? P.delta + static_cast<size_t>(1 - dir) * P.delta_stride
                    : (TR ? P.delta + static_cast<size_t>(dir) * P.delta_stride : nullptr);
    {
        u32x4 rc0[NT];
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            rc0[ct] = load_rec(c_begin, ct);
            rcA[ct] = load_rec(c_begin + 1, ct);
            rcX0[ct] = load_rec(c_begin + 2, ct);
            rcX1[ct] = rcX0[ct];
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                farp0[ct][t] = farp1[ct][t] = 0.0f;     // the first kRing + 1 chunks have no far sources
                mks0[ct][t] = mks1[ct][t] = 0;
                gs0[ct][t] = 0.0f;
                x0[ct][t] = xs0[ct][t] = xs1[ct][t] = 0.0f;
            }
        }
        const uint32_t info0 = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(rc0[0][3])));
        rows0 = rows_of(info0);
        p0 = __builtin_amdgcn_readfirstlane(static_cast<int>(rc0[0][2]));
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const int r = 4 * ct + kg;
            const int rr = r < rows0 ? r : 0;
            const uint32_t id = rc0[ct][3] & kRecNoNode;
            vg0[ct] = n0 + static_cast<int>(id == kRecNoNode ? 0u : id);
            if constexpr (FF) {
                ftp0[ct] = *reinterpret_cast<const f32x4 *>(featb + static_cast<uint32_t>(vg0[ct]));
                ftp1[ct] = ftp0[ct];
            } else {
                if constexpr (BW) {
                    load_cols(P.emb, static_cast<uint32_t>(vg0[ct] * 2 * H + (1 - dir) * H), xs0[ct]);
                    load_gates(gates_in, static_cast<uint32_t>(vg0[ct] * H), mks0[ct]);
                } else {
                    load_cols(xin, static_cast<uint32_t>((p0 + rr) * H), xs0[ct]);
                }
            }
        }
        __syncthreads();
        gather(info0, rc0, farp0, bit0, mks0, gs0);
    }
    __syncthreads();

    // rB / rC: records of chunk c + 2 / target of chunk c + 3's; fC / fN: feature records of chunk
    // c / target of chunk c + 1's; xC, mC / xN, mN: the same for residual inputs and gate bytes;
    // farA / farB: far messages of chunk c + 1 / target of chunk c + 2's
    auto step = [&](auto twoc, int c, u32x4 (&rB)[NT], u32x4 (&rC)[NT], f32x4 (&fC)[NT], f32x4 (&fN)[NT],
                    float (&xC)[NT][TPW], float (&xN)[NT][TPW], int (&mC)[NT][TPW], int (&mN)[NT][TPW],
                    float (&farA)[NT][TPW], float (&farB)[NT][TPW]) __attribute__((always_inline)) {
        const int rows = rows0;
        // the chunk fills a second row tile: known when the code is compiled (kind 0 / 1), or not (-1)
        constexpr int kind = decltype(twoc)::value;
        const bool two = kind < 0 ? rows > kTileNodes : kind > 0;
        const bool has_next = c + 1 < c_end;
        const int ring = static_cast<int>(static_cast<unsigned>(c - c_begin) % RING);   // table rows ring * CH .. of this chunk's messages
        const uint32_t info1 = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(rcA[0][3])));
        const int rows1 = rows_of(info1);
        const int p1 = __builtin_amdgcn_readfirstlane(static_cast<int>(rcA[0][2]));

        // Accumulators, one chain per (row tile, column tile): acc[ct][t].  The chains of a wave's
        // column tiles (and of the co-resident workgroup) interleave, so a dependent matrix
        // instruction never waits for its predecessor.
        f32x4 acc[2][TPW];
        int gate_bits[NT][TPW];   // (TR) ReLU gates of this chunk's rows, collected layer by layer

#pragma unroll
        for (int n = 0; n < NL; ++n) {
            // ---- rows of A from LDS (activation parts), weights from registers
            // One row tile: the A fragments are read first (a1), the loads and stores of the
            // pipeline ("mid block") are issued while they travel, then the matrix instructions.
            bf16x8 a1[KS];
            float bias_n[TPW];
#pragma unroll
            for (int t = 0; t < TPW; ++t) bias_n[t] = kBiasLds ? bias_row[n * H + mcol(t)] : bias[n][t];
            auto read_one_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    a1[ks] = *reinterpret_cast<const bf16x8 *>(act_at(n & 1, col, 32 * ks + 8 * kg));
            };
            auto mfma_one_tile = [&]() __attribute__((always_inline)) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
#pragma unroll
                        for (int ws = 0; ws < WS; ++ws) {
                            const f32x4 c_in = (ks == 0 && ws == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[0][t];
                            acc[0][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1[ks], W[n][t][ks][ws], c_in, 0, 0, 0);
                        }
                }
            };
            auto mfma_two_tiles = [&]() __attribute__((always_inline)) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        const bf16x8 a =
                            *reinterpret_cast<const bf16x8 *>(act_at(n & 1, 16 * ct + col, 32 * ks + 8 * kg));
#pragma unroll
                        for (int t = 0; t < TPW; ++t)
#pragma unroll
                            for (int ws = 0; ws < WS; ++ws) {
                                const f32x4 c_in = (ks == 0 && ws == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[ct][t];
                                acc[ct][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, W[n][t][ks][ws], c_in, 0, 0, 0);
                            }
                    }
            };
            // ---- epilogue: lane (col, kg) holds, for node 4 ct + kg and output column
            // wc0 + 16 t + col, the three partial products in rows 0..2 of its accumulators.
            // Row tile 0 is handled by code common to both kinds of chunk, so that its stores
            // are on every path (see sink_row).
            // `dead`: the row tile is beyond the chunk's rows (a chunk of one tile): nothing is
            // computed for it, but its global stores are issued all the same (to the sink rows),
            // so that both kinds of chunk leave the same number of stores behind every load.
            auto epilogue = [&](int ct, auto deadc) __attribute__((always_inline)) {
                constexpr bool dead = decltype(deadc)::value;
                const int r = ct * kTileNodes + kg;
                const bool live = !dead && r < rows;
                const int v_emb = live ? vg0[ct] : gv.n_tot;
                const int v_msg = live ? vg0[ct] : sink_row;
                // row of this node in the kept / delta array `slot` (unused rows: the spare row)
                auto delta_at = [&](int slot) __attribute__((always_inline)) {
                    return live ? static_cast<uint32_t>(slot * gv.n_tot * H) + static_cast<uint32_t>(vg0[ct] * H)
                                : static_cast<uint32_t>(2 * L * gv.n_tot * H);
                };
                float yv[TPW], ypre[TPW];
#pragma unroll
                for (int t = 0; t < TPW; ++t) yv[t] = dead ? 0.0f : acc[ct][t][0] + acc[ct][t][1] + acc[ct][t][2];
                if constexpr (BW) {
                    // delta slot of this layer's gated output: f's layers L-2 .. 0, then g's
                    // layers L-1 .. 0; slot = index into the 2L delta arrays (f first)
                    if (n == 0) {
                        float g[TPW];
#pragma unroll
                        for (int t = 0; t < TPW; ++t) g[t] = dead ? 0.0f : gs0[ct][t];
                        store_cols(dlt, delta_at(L - 1), g);
                    }
                    auto gate = [&](int bit) __attribute__((always_inline)) {
                        if constexpr (!dead) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) yv[t] = (mC[ct][t] & bit) ? yv[t] : 0.0f;
                        }
                    };
                    if (n == L - 1) {                // end of f^T: ds_v = outside gradient + f path
                        if constexpr (!dead) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) yv[t] += FF ? x0[ct][t] : xC[ct][t];
                        }
                        store_cols(P.emb, static_cast<uint32_t>(v_emb * 2 * H + (1 - dir) * H), yv);
                        gate(4);
                        store_cols(dlt, delta_at(L + L - 1), yv);
                    } else if (n < L - 1) {
                        gate(2);
                        store_cols(dlt, delta_at(L - 2 - n), yv);
                    } else if (n < NL - 1) {
                        gate(8);
                        store_cols(dlt, delta_at(L + NL - 2 - n), yv);
                    }
                    if (n == NL - 1) {               // end of g^T: da_v
                        store_cols(msg, static_cast<uint32_t>(v_msg * H), yv);
                        if constexpr (!dead) store_cols(msgtab, static_cast<uint32_t>((ring * CH + r) * LDM), yv);
                    }
                    if constexpr (!dead) {
                        if (n < NL - 1) put_rows((n + 1) & 1, r, yv);
                    }
                    return;
                }
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    float y = yv[t];
                    if constexpr (!dead) y = fmaxf(y + bias_n[t], 0.0f);
                    if constexpr (TR && !dead) {
                        const int bit = n == NL - 1 ? 1 : (n == L - 1 ? 4 : (n == 0 ? 8 : 2));
                        gate_bits[ct][t] = (n == 0 ? 0 : gate_bits[ct][t]) | (y > 0.0f ? bit : 0);
                    }
                    ypre[t] = y;
                    if (n == L - 1) {                    // end of g: residual update of s_v
                        if constexpr (!dead) y += FF ? x0[ct][t] : xC[ct][t];
                    }
                    if (n == NL - 1) {                   // end of f: the message of v, flagged
                        const uint32_t flag = (!dead && (bit0[ct] | (vg0[ct] == cur))) ? 0x80000000u : 0u;
                        y = __uint_as_float(__float_as_uint(y) | flag);
                    }
                    yv[t] = y;
                }
                // a forward sweep's stores to HBM: ypre = the layer's output, yv = what the layer
                // hands on (the state after the residual, the flagged message)
                auto hbm_stores = [&]() __attribute__((always_inline)) {
                    if constexpr (TR) {
                        // the output of g's last layer is only ever needed as a gate
                        if (n < NL - 1 && n != L - 1) store_cols(dlt, delta_at(1 + n), ypre);
                        if (n == NL - 1) {
                            int gb[TPW];
#pragma unroll
                            for (int t = 0; t < TPW; ++t) gb[t] = dead ? 0 : gate_bits[ct][t];
                            store_gates(gates_out, live ? static_cast<uint32_t>(vg0[ct] * H)
                                                        : static_cast<uint32_t>((2 - dir) * gv.n_tot * H), gb);
                        }
                    }
                    if (n == L - 1) {
                        store_cols(P.emb, static_cast<uint32_t>(v_emb * 2 * H + dir * H), yv);
                        if constexpr (WX) store_cols(xb, static_cast<uint32_t>((live ? n0 + p0 + r : spare_row) * H), yv);
                    }
                    if (n == NL - 1) store_cols(msg, static_cast<uint32_t>(v_msg * H), yv);
                };
                if constexpr (!kLdsFirst) hbm_stores();
                // What the next layer (or the next chunk's gather) waits for goes to LDS; where the
                // registers allow, before the stores to HBM, which then follow while the LDS
                // writes complete.
                if constexpr (!dead) {
                    if (n < NL - 1)
                        put_rows((n + 1) & 1, r, yv);
                    else
                        store_cols(msgtab, static_cast<uint32_t>((ring * CH + r) * LDM), yv);
                    if constexpr (kLdsFirst) __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (kLdsFirst) hbm_stores();
            };

            // The loads and stores of the pipeline (the "mid block" below) are issued while the A
            // fragments travel from LDS where a wave has the registers to hold the fragments
            // meanwhile (one column tile per wave); otherwise behind the matrix instructions.
            auto mid_block = [&]() __attribute__((always_inline)) {
                if (n == 0) {
                    // First layer: the far messages of chunk c + 2
                    // (this wave's columns, in the layout in which they are summed).  A row without
                    // a far source reads the row of zeros.  The messages were stored by this wave
                    // at least kRing - 1 chunks ago; see the note at the top of the file.
                    const uint32_t info2 = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(rB[0][3])));
                    const bool two2 = kLoadTile1Always || rows_of(info2) > kTileNodes;
                    float dterm[NT][TPW];
                    if constexpr (FF) {
#pragma unroll
                        for (int ct = 0; ct < NT; ++ct)
                            if (ct == 0 || two) {
#pragma unroll
                                for (int t = 0; t < TPW; ++t) dterm[ct][t] = device_term(fC[ct], t);
                            }
                    }
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct) {
                        if (ct > 0 && !two2) continue;
                        const uint32_t u = rB[ct][1];
                        const bool wanted = (rB[ct][0] & kRecListed) == 0 && u != kNoFar;
                        const int row = wanted ? n0 + static_cast<int>(u) : spare_row;
                        load_cols(msg, static_cast<uint32_t>(row * H), farB[ct]);
                    }
                    if constexpr (FF) {
#pragma unroll
                        for (int ct = 0; ct < NT; ++ct)
                            if (ct == 0 || two) {
#pragma unroll
                                for (int t = 0; t < TPW; ++t) x0[ct][t] = project(fC[ct], dterm[ct][t], t);
                            }
                    }
                }
                // The records of chunk c + 3 and the inputs of chunk c + 1: behind the second layer's
                // matrix instructions; in the reverse pass behind the first layer's, ahead of that
                // layer's stores: loads and stores retire in order, the reverse pass stores six times
                // per row and chunk, and a load queued behind a layer's stores returned too late for
                // the next chunk (2.35 -> 2.22 ms; no change for the forward sweeps).
                if (n == ((NL > 2 && !BW) ? 1 : 0)) {
                    const bool two1 = kLoadTile1Always || rows1 > kTileNodes;
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct) {
                        rC[ct] = load_rec(c + 3, ct);
                        if (ct > 0 && !two1) continue;
                        const int r = 4 * ct + kg;
                        const int rr = (r < rows1) ? r : 0;
                        if constexpr (FF) {
                            fN[ct] = *reinterpret_cast<const f32x4 *>(featb + static_cast<uint32_t>(node_of(rcA[ct])));
                        } else {
                            if constexpr (BW) {
                                const int v = node_of(rcA[ct]);
                                load_cols(P.emb, static_cast<uint32_t>(v * 2 * H + (1 - dir) * H), xN[ct]);
                                load_gates(gates_in, static_cast<uint32_t>(v * H), mN[ct]);
                            } else {
                                load_cols(xin + static_cast<size_t>(p1) * H, static_cast<uint32_t>(rr * H), xN[ct]);
                            }
                        }
                    }
                }

                if (n == NL - 1) {
                    // Last layer: the reachability bits of this
                    // chunk's nodes go to HBM (for the pooling kernel).
                    if constexpr (!BW) {
#pragma unroll
                        for (int ct = 0; ct < (kind == 0 ? 1 : NT); ++ct) {
                            const int r = ct * kTileNodes + kg;
                            const bool mine = wave == 0 && col == 0 && r < rows;
                            reach[static_cast<uint32_t>(mine ? vg0[ct] : sink_row)] = static_cast<uint8_t>(bit0[ct]);
                        }
                    }
                }

            };
            if constexpr (kReadFirst) {
                if (!two) read_one_tile();
                __builtin_amdgcn_sched_barrier(0);
                mid_block();
                __builtin_amdgcn_sched_barrier(0);
                if (two)
                    mfma_two_tiles();
                else
                    mfma_one_tile();
            } else {
                if (two) {
                    mfma_two_tiles();
                } else {
                    read_one_tile();
                    mfma_one_tile();
                }
                mid_block();
            }

            epilogue(0, std::false_type{});
            if constexpr (kind == 0 && kSinkStores)
                epilogue(1, std::true_type{});
            else if (two)
                epilogue(1, std::false_type{});

            // The table rows that chunk c + 1 sums were all written by this wave (its own
            // columns), so its gather follows without a barrier.
            if (n == NL - 1 && has_next) gather(info1, rcA, farA, bit0, mN, gs0);
            lds_barrier();
        }

        rows0 = rows1;
        p0 = p1;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            const uint32_t id = rcA[ct][3] & kRecNoNode;
            vg0[ct] = n0 + static_cast<int>(id == kRecNoNode ? 0u : id);
            rcA[ct] = rB[ct];       // arrived: its far ids were used behind this chunk's first layer
        }
    };
    // Both kinds of chunk (one row tile, two) are compiled as straight-line code of their own.
    // Nothing loaded before the loop is still in flight when it starts: the waits inside the loop
    // are then counted from the loop's own loads and stores alone (a load issued just before the
    // loop would otherwise make every iteration wait for all but its newest memory operation).
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
    using one_tile = std::integral_constant<int, 0>;
    using two_tiles = std::integral_constant<int, 1>;
    using either = std::integral_constant<int, -1>;
    for (int c = c_begin; c < c_end; c += 2) {
        if constexpr (!kSplitKinds) {
            step(either{}, c, rcX0, rcX1, ftp0, ftp1, xs0, xs1, mks0, mks1, farp0, farp1);
            if (c + 1 < c_end) step(either{}, c + 1, rcX1, rcX0, ftp1, ftp0, xs1, xs0, mks1, mks0, farp1, farp0);
            continue;
        }
        if (rows0 > kTileNodes)
            step(two_tiles{}, c, rcX0, rcX1, ftp0, ftp1, xs0, xs1, mks0, mks1, farp0, farp1);
        else
            step(one_tile{}, c, rcX0, rcX1, ftp0, ftp1, xs0, xs1, mks0, mks1, farp0, farp1);
        if (c + 1 < c_end) {
            if (rows0 > kTileNodes)
                step(two_tiles{}, c + 1, rcX1, rcX0, ftp1, ftp0, xs1, xs0, mks1, mks0, farp1, farp0);
            else
                step(one_tile{}, c + 1, rcX1, rcX0, ftp1, ftp0, xs1, xs0, mks1, mks0, farp1, farp0);
        }
    }
}

// Raw features of every node as one 16-byte record (Section 2.1 features; the device and the
// is-current flag travel as bits), in node order: a sweep reads a row's record by the node id that
// the row's plan record names, one chunk ahead.
__global__ __launch_bounds__(256) void k_feature_records(GraphView gv, const float *__restrict__ feats,
                                                      const int32_t *__restrict__ placement,
                                                      const int32_t *__restrict__ cur_node, int D,
                                                      float4 *__restrict__ featb)
{
    const int v = blockIdx.x * 256 + threadIdx.x;
    if (v >= gv.n_tot) return;
    const int b = gv.node_graph[v];
    const int dev = placement[v];
    const int bits = ((dev >= 0 && dev < D) ? dev : 0xFFFF) | ((v - gv.node_off[b] == cur_node[b]) ? 0x10000 : 0);
    const float4 rec{feats[v * 3 + 0], feats[v * 3 + 1], feats[v * 3 + 2], __int_as_float(bits)};
    featb[v] = rec;
}

}  // namespace

// Packs the f and g weights of both directions into MFMA B-operand fragments.
// Index: ((((dir * 2L + n) * MT + mt) * KS + ks) * WS + ws) * 64 + lane, n = g layers then f
// layers; lane l holds W[k(ks, l / 16, i)][16 mt + l % 16], i = 0..7, as bf16 part ws of the
// exact three-way split (ws = 0 only when the weights are bf16 already).  k is the position of
// an input column in the kernel's activation rows, 32 ks + 8 (l / 16) + i.  Where a wave owns two
// column tiles (H = 128) they interleave: tile mt holds the columns 32 (mt / 2) + 2 c + mt % 2,
// c = 0..15, so that a lane's two columns are neighbours (see mcol in the kernel).
// With `reverse`, the fragments of the reverse pass: index dir is the direction whose chunks are
// walked, the weights are those of the other direction, transposed, f's layers from the last to
// the first and then g's (biases are not used there).
void pack_sweep_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                        std::vector<float> *bias, bool reverse)
{
    const int H = mv.H, L = mv.L, MT = H / 16, KS = H / 32, NL = 2 * L;
    const bool paired = MT / sweep_waves(H) == 2;
    frag->assign(static_cast<size_t>(2) * NL * MT * KS * WS * 64 * 8, 0);
    bias->assign(static_cast<size_t>(2) * NL * H, 0.0f);
    auto to_bf16 = [](float x) {
        uint32_t u;
        std::memcpy(&u, &x, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return static_cast<uint16_t>(u >> 16);
    };
    auto from_bf16 = [](uint16_t h) {
        uint32_t u = static_cast<uint32_t>(h) << 16;
        float x;
        std::memcpy(&x, &u, 4);
        return x;
    };
    for (int dir = 0; dir < 2; ++dir)
        for (int n = 0; n < NL; ++n) {
            const LayerRef &lr = reverse ? ((n < L) ? mv.f[1 - dir].layer[L - 1 - n] : mv.g[1 - dir].layer[NL - 1 - n])
                                         : ((n < L) ? mv.g[dir].layer[n] : mv.f[dir].layer[n - L]);
            for (int h = 0; h < H; ++h)
                (*bias)[(static_cast<size_t>(dir) * NL + n) * H + h] = reverse ? 0.0f : blob[lr.b + h];
            for (int mt = 0; mt < MT; ++mt)
                for (int ks = 0; ks < KS; ++ks)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int i = 0; i < 8; ++i) {
                            const int k = 32 * ks + 8 * (lane / 16) + i;
                            const int m = paired ? 32 * (mt / 2) + 2 * (lane % 16) + mt % 2 : 16 * mt + lane % 16;
                            float rest = reverse ? blob[lr.w + static_cast<size_t>(m) * H + k]
                                                 : blob[lr.w + static_cast<size_t>(k) * H + m];
                            for (int ws = 0; ws < WS; ++ws) {
                                const uint16_t part = to_bf16(rest);
                                rest -= from_bf16(part);
                                const size_t at =
                                    (((((static_cast<size_t>(dir) * NL + n) * MT + mt) * KS + ks) * WS + ws) * 64 + lane) * 8 + i;
                                (*frag)[at] = part;
                            }
                        }
        }
}

bool sweep_mfma_supported(int H, int L, int weight_dtype)
{
    if (L < 1 || L > 2) return false;
    if (weight_dtype == PL_WEIGHTS_BF16) return H == 32 || H == 64 || H == 128;
    return H == 32 || H == 64;
}

void launch_sweep_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                       const ForwardArgs &fa, const uint4 *wfrag, const float *bias, int WS,
                       bool first_sweep, bool more_sweeps, float *keep, size_t keep_stride, uint8_t *gates,
                       hipStream_t s)
{
    if (gv.B == 0) return;
    // keep, gates: where a single sweep also stores a_v, the layer outputs and the ReLU gates for the
    // reverse pass (TR)
    const bool tr = keep && gates && first_sweep && !more_sweeps;
    SweepParams P{gv, wfrag, bias, ws.emb, ws.xb, ws.msg, ws.reach, fa.cur_node,
                  ws.featb, first_sweep ? mv.blob + mv.proj.w : nullptr, mv.D, tr ? gates : nullptr,
                  tr ? keep : nullptr, tr ? keep_stride : 0};
    if (first_sweep)
        hipLaunchKernelGGL(k_feature_records, dim3((gv.n_tot + 255) / 256), dim3(256), 0, s, gv, fa.node_feats,
                           fa.placement, fa.cur_node, mv.D, ws.featb);
    const dim3 grid(2 * gv.B);
#define PL_CASE(HH, WW, LL)                                                      \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                  \
        const dim3 block(64 * sweep_waves(HH));                                  \
        if (tr)                                                                  \
            hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, true, false, false, true>), grid, block, 0, s, P); \
        else if (first_sweep && more_sweeps)                                     \
            hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, true, true>), grid, block, 0, s, P);   \
        else if (first_sweep)                                                    \
            hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, true, false>), grid, block, 0, s, P);  \
        else if (more_sweeps)                                                    \
            hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, false, true>), grid, block, 0, s, P);  \
        else                                                                     \
            hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, false, false>), grid, block, 0, s, P); \
        return;                                                                  \
    }
    PL_CASE(128, 1, 2) PL_CASE(128, 1, 1)
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
}

// The reverse pass of one sweep in both directions (see BW at the kernel).  demb [n_tot + 1, 2H]
// holds the outside gradient of every state on entry and the gradient of the sweep's input on
// return; mask4 the gate bytes of both sweep directions in node order; dagg [2 n_tot + 2, H] must
// have its row 2 n_tot zero.
void launch_sweep_mfma_bw(const GraphView &gv, const ModelView &mv, const uint4 *wfrag, const float *bias,
                          int WS, const int32_t *cur_node, float *demb, float *dagg, uint8_t *mask4,
                          float *delta, size_t delta_stride, hipStream_t s)
{
    if (gv.B == 0) return;
    SweepParams P{gv, wfrag, bias, demb, nullptr, dagg, nullptr, cur_node, nullptr, nullptr, mv.D,
                  mask4, delta, delta_stride};
    const dim3 grid(2 * gv.B);
#define PL_CASE(HH, WW, LL)                                                                  \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                              \
        hipLaunchKernelGGL((k_sweep_mfma<HH, WW, LL, false, false, true>), grid,             \
                           dim3(64 * sweep_waves(HH)), 0, s, P);                             \
        return;                                                                              \
    }
    PL_CASE(128, 1, 2) PL_CASE(128, 1, 1)
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
}

}  // namespace pl
