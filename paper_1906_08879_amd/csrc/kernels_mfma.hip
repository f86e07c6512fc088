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
//   * A wave owns its output columns from end to end: it writes its columns of a message into
//     an LDS table, stages its columns of older messages (prefetched from HBM one chunk ahead)
//     into the same table, and sums its columns for the next chunk, in the MFMA result layout
//     (lane = node of the tile, column).  The table therefore needs no barrier; only the A
//     rows of the next layer cross waves: one LDS barrier per layer, four per chunk.
//   * Messages are ReLU outputs, so in the table their sign bit carries the reachability flag
//     of Section 2.2 step 3 (the node is v* or was computed from v*): sums take |x| and OR the
//     signs.  Row records name a fixed number of table slots (unused ones a zero row), so the
//     common gather is branch-free.
//   * On the first sweep the same lane computes its columns of x_v = relu(W_in^T phi_v + b)
//     (step 1) from the node's 16-byte feature record: x never exists in HBM.
//   * Barriers order LDS traffic only, so global prefetches stay in flight across them.
//     A message written to HBM in chunk c is only read back from HBM from chunk c + 3 on
//     (nearer consumers use the LDS table); by then the store has retired, because each
//     wave waits once per chunk for a batch of loads that it issued after that store.
//     Every global store is on every path (unused rows store to sink rows), so the number of
//     stores behind a load is known at compile time and waiting for the load never waits for
//     the stores.
//   * The kernel runs a dependent chain (about a thousand chunks of four layers per graph),
//     so it is bound by LDS round trips, MFMA latency and barriers, not by HBM bandwidth.
#include <type_traits>

#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int CH = kChunkRows, FCAP = kFarCap, RING = kRing;
constexpr int kTileNodes = 4;                 // nodes per 16-row MFMA tile (hi, mid, lo, zero rows)
constexpr int NT = CH / kTileNodes;           // row tiles per chunk

// Workgroup barrier that orders LDS traffic only: global prefetches stay outstanding.
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
    // here from the node's raw features, kept in bucket order, 16 bytes per node
    const float4 *featb;    // [2, n_tot] {run time, output size, is-visited, bits(device | is-current << 16)}
    const float *proj;      // [(F + 1), H]: rows of W_in, then b_in; NULL when the input comes from xb
    int D;
    // reverse pass (BW): ReLU masks of the node's layers in bucket order, one byte per (node,
    // column): bit 0 gates the gathered sum, bits 1..3 the outputs of layers 0 (L = 2 only),
    // L - 1 and L (L = 2 only); and the layer deltas, 2L arrays [n_tot, H] in node order
    const uint8_t *mask4;   // [2, n_tot, H]
    float *delta;           // per sweep direction: [2L][n_tot, H] (f's layers, then g's), then H
                            // floats that take the stores of a chunk's unused rows
    size_t delta_stride;    // floats between the two directions' blocks
};

// Reads a chunk's meta record through the constant address space, so that the wave-uniform
// record comes in with a scalar load.
typedef int i32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4 load_uniform(const int4 *p)
{
    const i32x4 r = *reinterpret_cast<const __attribute__((address_space(4))) i32x4 *>(
        reinterpret_cast<uintptr_t>(p));
    return int4{r.x, r.y, r.z, r.w};
}

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
// stored gates, table entries are signed (no reachability flag), and every gated layer input
// is also written to HBM as the layer's delta for the weight gradients.
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
    constexpr int LDA = H + 8;                 // bf16 row stride of the activation buffers
    constexpr int LDM = H + 16;                // float row stride of the message table (16 mod 64:
                                               // four consecutive rows fall on disjoint banks)
    constexpr int QW = WC / 4;                 // float4 per far row and wave
    constexpr int PFN = (FCAP * QW + 63) / 64; // staged far float4 per lane
    constexpr int NACC = KS > 1 ? 2 : 1;       // independent accumulation chains per tile
    constexpr int kZeroSlot = kMsgSlots;
    constexpr int kWarmAhead = 12;             // chunks between touching a chunk record and reading it
    static_assert(NTL % NW == 0, "column tiles must divide over the waves");

    // Message table: H floats per row.  Messages are ReLU outputs, so their sign bit is free:
    // in the table it carries the reachability flag of the row's node (set if the node is v* or
    // has v* among the nodes it was computed from); sums take |x|.  A wave reads and writes
    // only its own columns, so the table needs no barrier.  The last row stays zero.
    __shared__ __attribute__((aligned(16))) float msgtab[(kMsgSlots + 1) * LDM];
    __shared__ __attribute__((aligned(16))) __bf16 actbuf[2][NT * 16][LDA];
    __shared__ float proj_dev[(kMaxD + 1) * H];   // one-hot device rows of W_in, then a zero row

    const int b = blockIdx.x >> 1, dir = blockIdx.x & 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;    // MFMA result: column col, node kg of a tile
    const int wc0 = wave * WC;

    const GraphView &gv = P.gv;
    const SweepPlanView plan = gv.plan[dir];
    const int32_t *order = gv.order[dir];
    float *msg = P.msg + static_cast<size_t>(dir) * gv.n_tot * H;
    float *xb = P.xb + static_cast<size_t>(dir) * gv.n_tot * H;
    uint8_t *reach = P.reach + static_cast<size_t>(dir) * gv.n_tot;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = P.cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const int c_begin = plan.ck_off[b], c_end = plan.ck_off[b + 1];
    if (c_begin >= c_end) return;
    // one row past both directions' messages (and one byte past both directions' bits) is
    // never written: the address of dummy loads, relative to this direction's base.  The row
    // (byte) after it, and row n_tot of emb, take the stores of a chunk's unused rows: every
    // lane stores on every chunk, so the number of stores in flight behind a load is known
    // when the kernel is compiled and a wait for that load does not wait for the stores.
    const int spare_row = (2 - dir) * gv.n_tot;
    const int sink_row = spare_row + 1;

    // ---- weights of this direction into registers (B operand: lane holds column 16 nt + col)
    bf16x8 W[NL][TPW][KS][WS];
    float bias[NL][TPW];
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
            bias[n][t] = P.bias[(static_cast<size_t>(dir) * NL + n) * H + nt * 16 + col];
        }

    // ---- input projection (Section 2.2 step 1), one output column per lane and tile:
    // x = relu(b + time w0 + size w1 + w[2 + device] + is_current w[2 + D] + visited w[3 + D])
    const int D = P.D;
    float pw_time[TPW], pw_size[TPW], pw_cur[TPW], pw_vis[TPW], pw_b[TPW];
    if constexpr (FF) {
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int m = wc0 + 16 * t + col;
            pw_time[t] = P.proj[m];
            pw_size[t] = P.proj[H + m];
            pw_cur[t] = P.proj[(2 + D) * H + m];
            pw_vis[t] = P.proj[(3 + D) * H + m];
            pw_b[t] = P.proj[(4 + D) * H + m];
        }
        for (int i = tid; i < (kMaxD + 1) * H; i += kThreads)
            proj_dev[i] = (i < D * H) ? P.proj[2 * H + i] : 0.0f;
    }
    const float4 *featb = P.featb + static_cast<size_t>(dir) * gv.n_tot;
    // the device's row of W_in comes from LDS: read early (device_term), used late (project)
    auto device_term = [&](const f32x4 ft, int t) {
        const int dev = __float_as_int(ft[3]) & 0xFFFF;
        return proj_dev[(dev < D ? dev : D) * H + wc0 + 16 * t + col];
    };
    auto project = [&](const f32x4 ft, float dev_term, int t) {
        const int bits = __float_as_int(ft[3]);
        float o = pw_b[t];
        o = fmaf(ft[0], pw_time[t], o);
        o = fmaf(ft[1], pw_size[t], o);
        o += dev_term;
        o += (bits >> 16) ? pw_cur[t] : 0.0f;
        return fmaxf(fmaf(ft[2], pw_vis[t], o), 0.0f);
    };
    for (int i = tid; i < (kMsgSlots + 1) * LDM; i += kThreads) msgtab[i] = 0.0f;
    for (int i = tid; i < 2 * NT * 16 * LDA; i += kThreads) (&actbuf[0][0][0])[i] = static_cast<__bf16>(0.0f);

    // Writes y, split exactly into three bf16 parts, as rows 4 r .. 4 r + 2 of an A operand.
    auto put_parts = [&](int buf, int r, int m, float y) {
        const float rr = y - trunc_bf16(y);
        const float ll = rr - trunc_bf16(rr);
        unsigned short *dst = reinterpret_cast<unsigned short *>(&actbuf[buf][4 * r][m]);
        dst[0] = static_cast<unsigned short>(__float_as_uint(y) >> 16);
        dst[LDA] = static_cast<unsigned short>(__float_as_uint(rr) >> 16);
        dst[2 * LDA] = static_cast<unsigned short>(__float_as_uint(ll) >> 16);
    };

    // ---- gather of a chunk: a_v = sum of neighbour messages, for rows kg and kg + 4 and this
    // wave's columns, from the wave's own part of the LDS table; written as A rows of the first
    // layer.  K entries of every row record are summed (unused entries name the zero row).
    // Reverse pass: the sum is gated by bit 0 of the row's mask and kept in gs (it is the delta
    // of f's last layer, stored when the chunk is processed).
    auto gather_fixed = [&](auto kc, int ntile_x, const u32x4 (&ent)[NT], int (&bit)[NT],
                            const int (&mk)[NT][TPW], float (&gs)[NT][TPW]) {
        constexpr int K = decltype(kc)::value;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            bit[ct] = 0;
            if (ct >= ntile_x) continue;
            const u32x4 rec = ent[ct];
            float s[TPW];
            uint32_t signs = 0;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int slot = static_cast<int>((rec[k / 5] >> (6 * (k % 5))) & 63u);
                const float *row = msgtab + slot * LDM;
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const float x = row[wc0 + 16 * t + col];
                    const float ax = BW ? x : fabsf(x);
                    s[t] = k == 0 ? ax : s[t] + ax;
                    if (!BW && t == 0) signs |= __float_as_uint(x);
                }
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if constexpr (BW) {
                    s[t] = (mk[ct][t] & 1) ? s[t] : 0.0f;
                    gs[ct][t] = s[t];
                }
                if constexpr (TR) gs[ct][t] = s[t];
                put_parts(0, 4 * ct + kg, wc0 + 16 * t + col, s[t]);
            }
            bit[ct] = static_cast<int>(signs >> 31);
        }
    };
    // The same for a chunk in which some row has more neighbours than its record holds: that
    // row sums a list of table slots (recent sources) and node ids (sources at least three
    // chunks back, read from HBM).
    auto gather_general = [&](int ntile_x, const u32x4 (&ent)[NT], int (&bit)[NT],
                              const int (&mk)[NT][TPW], float (&gs)[NT][TPW]) {
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            bit[ct] = 0;
            if (ct >= ntile_x) continue;
            const u32x4 rec = ent[ct];
            const bool listed = ((rec[0] >> 30) & 1u) != 0;
            float s[TPW];
            uint32_t signs = 0;
#pragma unroll
            for (int t = 0; t < TPW; ++t) s[t] = 0.0f;
#pragma unroll
            for (int k = 0; k < kMaxEnt; ++k) {
                const int raw = static_cast<int>((rec[k / 5] >> (6 * (k % 5))) & 63u);
                const float *row = msgtab + (listed ? kZeroSlot : raw) * LDM;
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const float x = row[wc0 + 16 * t + col];
                    s[t] += BW ? x : fabsf(x);
                    if (!BW) signs |= __float_as_uint(x);
                }
            }
            if (listed) {
                const int d0 = static_cast<int>(rec[1]);
                const int d1 = d0 + static_cast<int>(rec[2]);
                // The list is walked in passes of PB entries, three passes per step.  The sixteen
                // lanes of the row's group first load the step's entries (one load each per
                // pass, all in flight together) and hand them round with lane shuffles; then a
                // pass issues all its loads before the first use.  An entry is a table slot or a
                // node id; the other source of the pair is the table's zero row or the spare
                // (all-zero, never written) row of msg, so both are always read and added, in
                // list order.
                constexpr int PB = 16;
                if constexpr (TPW == 1)
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
                        int u[PB];
                        float xl[PB][TPW], xg[PB][TPW];
                        int rg[PB];
#pragma unroll
                        for (int k = 0; k < PB; ++k) {
                            u[k] = __shfl(idv[q], (lane & 48) + k);
                            const float *row = msgtab + (u[k] < 0 ? -1 - u[k] : kZeroSlot) * LDM;
                            const int v = u[k] >= 0 ? u[k] : spare_row;
#pragma unroll
                            for (int t = 0; t < TPW; ++t) {
                                xl[k][t] = row[wc0 + 16 * t + col];
                                xg[k][t] = msg[static_cast<uint32_t>(v * H + wc0 + 16 * t + col)];
                            }
                            rg[k] = BW ? 0 : reach[static_cast<uint32_t>(v)];
                        }
#pragma unroll
                        for (int k = 0; k < PB; ++k) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) {
                                s[t] += (BW ? xl[k][t] : fabsf(xl[k][t])) + xg[k][t];
                                if (!BW) signs |= __float_as_uint(xl[k][t]);
                            }
                            if (!BW) signs |= ((u[k] >= 0) & ((u[k] == cur) | (rg[k] != 0))) ? 0x80000000u : 0u;
                        }
                    }
                }
                // two column tiles per wave leave no registers for that: four entries at a time
                if constexpr (TPW > 1)
                for (int p = d0; p < d1; p += 4) {
                    int u[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) u[k] = p + k < d1 ? plan.ovf[p + k] : -1 - kZeroSlot;
                    float xl[4][TPW], xg[4][TPW];
                    int rg[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float *row = msgtab + (u[k] < 0 ? -1 - u[k] : kZeroSlot) * LDM;
                        const int v = u[k] >= 0 ? u[k] : spare_row;
#pragma unroll
                        for (int t = 0; t < TPW; ++t) {
                            xl[k][t] = row[wc0 + 16 * t + col];
                            xg[k][t] = msg[static_cast<uint32_t>(v * H + wc0 + 16 * t + col)];
                        }
                        rg[k] = BW ? 0 : reach[static_cast<uint32_t>(v)];
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
#pragma unroll
                        for (int t = 0; t < TPW; ++t) {
                            s[t] += (BW ? xl[k][t] : fabsf(xl[k][t])) + xg[k][t];
                            if (!BW) signs |= __float_as_uint(xl[k][t]);
                        }
                        if (!BW) signs |= ((u[k] >= 0) & ((u[k] == cur) | (rg[k] != 0))) ? 0x80000000u : 0u;
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                if constexpr (BW) {
                    s[t] = (mk[ct][t] & 1) ? s[t] : 0.0f;
                    gs[ct][t] = s[t];
                }
                if constexpr (TR) gs[ct][t] = s[t];
                put_parts(0, 4 * ct + kg, wc0 + 16 * t + col, s[t]);
            }
            bit[ct] = static_cast<int>(signs >> 31);
        }
    };
    // w = meta.w of the chunk: most entries of a row | (a row uses the list) << 8
    auto gather = [&](int w, int ntile_x, const u32x4 (&ent)[NT], int (&bit)[NT], const int (&mk)[NT][TPW],
                      float (&gs)[NT][TPW]) {
        if (w <= 2)
            gather_fixed(std::integral_constant<int, 2>{}, ntile_x, ent, bit, mk, gs);
        else if (w <= 5)
            gather_fixed(std::integral_constant<int, 5>{}, ntile_x, ent, bit, mk, gs);
        else if (w <= kMaxEnt)
            gather_fixed(std::integral_constant<int, kMaxEnt>{}, ntile_x, ent, bit, mk, gs);
        else
            gather_general(ntile_x, ent, bit, mk, gs);
    };

    // ---- software pipeline state.  m0 describes chunk c, m1 chunk c + 1.  A lane works on
    // rows kg (tile 0) and kg + 4 (tile 1) of a chunk.
    auto clampc = [&](int c) { return c < c_end ? c : c_end - 1; };
    int4 m0 = load_uniform(plan.meta + c_begin);
    int4 m1 = load_uniform(plan.meta + clampc(c_begin + 1));
    u32x4 ent1[NT];          // neighbour records of the rows of the chunk gathered next
    int vg0[NT], vg1[NT];    // node ids of the rows of chunk c, c + 1
    f32x4 ft0[NT];           // raw-feature records of the rows of chunk c        (FF)
    float x0[NT][TPW];       // residual inputs x_v of chunk c
    float x1[NT][TPW];       // ... of chunk c + 1                                  (!FF)
    int bit0[NT];            // reachability bits of the rows of chunk c
    int fid1[PFN];           // far sources of chunk c + 1
    int mk0[NT][TPW], mk1[NT][TPW];   // (BW) gate bytes of the rows of chunk c, c + 1
    float gs0[NT][TPW];      // (BW) gated gathered sums of chunk c: the delta of f's last layer
    const uint8_t *mask4 = BW ? P.mask4 + static_cast<size_t>(dir) * gv.n_tot * H : nullptr;
    float *dlt = BW ? P.delta + static_cast<size_t>(1 - dir) * P.delta_stride
                    : (TR ? P.delta + static_cast<size_t>(dir) * P.delta_stride : nullptr);
#pragma unroll
    for (int ct = 0; ct < NT; ++ct)
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            mk0[ct][t] = mk1[ct][t] = 0;
            gs0[ct][t] = 0.0f;
        }
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        const int r = 4 * ct + kg;
        const int rr = r < m0.y ? r : 0;
        ent1[ct] = *reinterpret_cast<const u32x4 *>(plan.ent + static_cast<size_t>(c_begin) * CH + r);
        vg0[ct] = order[m0.x + rr];
        vg1[ct] = vg0[ct];
        if constexpr (FF) {
            ft0[ct] = *reinterpret_cast<const f32x4 *>(featb + m0.x + rr);
        } else {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                x0[ct][t] = xb[static_cast<size_t>(m0.x + rr) * H + wc0 + 16 * t + col];
                x1[ct][t] = x0[ct][t];
                if constexpr (BW) {
                    mk0[ct][t] = mask4[static_cast<size_t>(m0.x + rr) * H + wc0 + 16 * t + col];
                    mk1[ct][t] = mk0[ct][t];
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < PFN; ++i) {
        const int f = (lane + 64 * i) / QW;
        fid1[i] = (f < FCAP) ? plan.far[static_cast<size_t>(clampc(c_begin + 1)) * FCAP + f] : -1;
    }
    __syncthreads();
    gather(m0.w, (m0.y + kTileNodes - 1) / kTileNodes, ent1, bit0, mk0, gs0);
    // every load so far has returned before the loop is entered (inside the loop the compiler
    // then never waits for more than the loads of the loop's own batch)
#pragma unroll
    for (int i = 0; i < PFN; ++i) asm volatile("" ::"v"(fid1[i]));
#pragma unroll
    for (int ct = 0; ct < NT; ++ct) {
        asm volatile("" ::"v"(vg0[ct]), "v"(vg1[ct]));
        if constexpr (FF) {
            asm volatile("" ::"v"(ft0[ct][0]));
        } else {
#pragma unroll
            for (int t = 0; t < TPW; ++t) asm volatile("" ::"v"(x0[ct][t]), "v"(x1[ct][t]));
            if constexpr (BW) {
#pragma unroll
                for (int t = 0; t < TPW; ++t) asm volatile("" ::"v"(mk0[ct][t]), "v"(mk1[ct][t]));
            }
        }
    }
    __syncthreads();

    for (int c = c_begin; c < c_end; ++c) {
        const int rows = m0.y;
        const bool two = rows > kTileNodes;      // the chunk fills a second row tile
        const bool has_next = c + 1 < c_end;
        const int par = (c - c_begin) & 1;

        // Plain vector types on purpose: arrays of the HIP float4 class that are written in one
        // unrolled branch and read in another are not always split into registers.
        f32x4 pf[PFN];           // far messages of chunk c + 1, in flight during the later layers
        int pf_reach[PFN];
        bool pf_cur[PFN];
        int4 m2 = m1;
        int warm = 0;            // see the prefetch of the chunk records below
        // Accumulators: a chunk of one row tile splits its k-steps over two chains per column
        // tile (acc[chain][t]); a chunk of two row tiles runs one chain per (row tile, column
        // tile) (acc[ct][t]): four independent chains either way.
        f32x4 acc[2][TPW];

#pragma unroll
        for (int n = 0; n < NL; ++n) {
            // ---- rows of A from LDS (activation parts), weights from registers
            auto mfma_one_tile = [&]() {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&actbuf[n & 1][col][32 * ks + 8 * kg]);
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
#pragma unroll
                        for (int ws = 0; ws < WS; ++ws) {
                            const f32x4 c_in = (ks < NACC && ws == 0) ? f32x4{0.f, 0.f, 0.f, 0.f} : acc[ks % NACC][t];
                            acc[ks % NACC][t] =
                                __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, W[n][t][ks][ws], c_in, 0, 0, 0);
                        }
                }
                if constexpr (NACC == 1) {
#pragma unroll
                    for (int t = 0; t < TPW; ++t) acc[1][t] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
            };
            auto mfma_two_tiles = [&]() {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        const bf16x8 a =
                            *reinterpret_cast<const bf16x8 *>(&actbuf[n & 1][16 * ct + col][32 * ks + 8 * kg]);
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
            // wc0 + 16 t + col, the three partial products in rows 0..2 of its accumulators
            // Row tile 0 is handled by code common to both kinds of chunk, so that its stores
            // are on every path (see sink_row).
            auto epilogue = [&](int ct) {
                const int r = ct * kTileNodes + kg;
                const bool live = r < rows;
                const int v_emb = live ? vg0[ct] : gv.n_tot;
                const int v_msg = live ? vg0[ct] : sink_row;
#pragma unroll
                for (int t = 0; t < TPW; ++t) {
                    const int m = wc0 + 16 * t + col;
                    float y = acc[ct][t][0] + acc[ct][t][1] + acc[ct][t][2];
                    if (ct == 0) {                       // one row tile: acc[1] is the second chain
                        const float y1 = acc[1][t][0] + acc[1][t][1] + acc[1][t][2];
                        y += two ? 0.0f : y1;
                    }
                    if constexpr (BW) {
                        // delta slot of this layer's gated output: f's layers L-2 .. 0, then g's
                        // layers L-1 .. 0; slot = index into the 2L delta arrays (f first)
                        const uint32_t d_row = live ? static_cast<uint32_t>(vg0[ct] * H + m)
                                                    : static_cast<uint32_t>(2 * L * gv.n_tot * H + m);
                        auto put_delta = [&](int slot, float val) {
                            dlt[live ? static_cast<uint32_t>(slot * gv.n_tot * H) + d_row : d_row] = val;
                        };
                        if (n == 0) put_delta(L - 1, gs0[ct][t]);
                        if (n == L - 1) {                // end of f^T: ds_v = outside gradient + f path
                            y += x0[ct][t];
                            P.emb[static_cast<uint32_t>(v_emb * 2 * H + (1 - dir) * H + m)] = y;
                            y = (mk0[ct][t] & 4) ? y : 0.0f;
                            put_delta(L + L - 1, y);
                        } else if (n < L - 1) {
                            y = (mk0[ct][t] & 2) ? y : 0.0f;
                            put_delta(L - 2 - n, y);
                        } else if (n < NL - 1) {
                            y = (mk0[ct][t] & 8) ? y : 0.0f;
                            put_delta(L + NL - 2 - n, y);
                        }
                        if (n == NL - 1) {               // end of g^T: da_v
                            msg[static_cast<uint32_t>(v_msg * H + m)] = y;
                            msgtab[(par * CH + r) * LDM + m] = y;
                        } else {
                            put_parts((n + 1) & 1, r, m, y);
                        }
                        continue;
                    }
                    y = fmaxf(y + bias[n][t], 0.0f);
                    if constexpr (TR) {
                        const uint32_t d_row = live ? static_cast<uint32_t>(vg0[ct] * H + m)
                                                    : static_cast<uint32_t>(2 * L * gv.n_tot * H + m);
                        if (n == 0) dlt[d_row] = gs0[ct][t];
                        if (n < NL - 1) dlt[live ? static_cast<uint32_t>((1 + n) * gv.n_tot * H) + d_row : d_row] = y;
                    }
                    if (n == L - 1) {                    // end of g: residual update of s_v
                        y += x0[ct][t];
                        P.emb[static_cast<uint32_t>(v_emb * 2 * H + dir * H + m)] = y;
                        if constexpr (WX) xb[static_cast<uint32_t>((live ? m0.x + r : spare_row) * H + m)] = y;
                    }
                    if (n == NL - 1) {                   // end of f: the message of v
                        msg[static_cast<uint32_t>(v_msg * H + m)] = y;
                        const uint32_t flag = (bit0[ct] | (vg0[ct] == cur)) ? 0x80000000u : 0u;
                        msgtab[(par * CH + r) * LDM + m] = __uint_as_float(__float_as_uint(y) | flag);
                    } else {
                        put_parts((n + 1) & 1, r, m, y);
                    }
                }
            };

            if (two)
                mfma_two_tiles();
            else
                mfma_one_tile();

            if (n == 0) {
                // The inputs of this chunk's residual, then the loads for the next chunk, issued
                // behind the first layer's matrix instructions.  The loads may read messages
                // that this workgroup stored to HBM at least two chunks ago.  Those stores are
                // complete: vector memory operations of a wave retire in order, and every wave
                // waited for its own previous batch of these loads (issued after those stores)
                // before the last barrier of the previous chunk.
                // Work for a second row tile (rows 4..7) is skipped when the chunk has none, and
                // far rows beyond the first 64 / QW only when the next chunk stages that many.
                float dterm[NT][TPW];
                if constexpr (FF) {
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct)
                        if (ct == 0 || two) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) dterm[ct][t] = device_term(ft0[ct], t);
                        }
                }
#pragma unroll
                for (int i = 0; i < PFN; ++i) {
                    if (i > 0 && m1.z <= i * (64 / QW)) continue;
                    const int e = lane + 64 * i;
                    const int f = e / QW, q = e - f * QW;
                    const bool wanted = has_next && f < m1.z && fid1[i] >= 0;
                    // lanes without a far source read a spare row that is never written, so
                    // that every wave has a load of this batch to wait for
                    const int u = wanted ? fid1[i] : spare_row;
                    pf[i] = *reinterpret_cast<const f32x4 *>(msg + static_cast<uint32_t>(u * H + wc0 + 4 * q));
                    pf_reach[i] = BW ? 0 : reach[static_cast<uint32_t>(u)];   // combined with pf_cur at the end of the chunk
                    pf_cur[i] = wanted && u == cur;
                }
                // The chunk records come in through the scalar cache, and a scalar load cannot be
                // overlapped with LDS work: every wait for LDS data also waits for the scalar loads
                // in flight.  So a vector load touches the record of a chunk some way ahead (its
                // value is not used): the scalar load of that record then finds its line in L2
                // instead of going to HBM every fourth chunk.
                {
                    int opaque = 0;
                    asm volatile("" : "+v"(opaque));
                    warm = reinterpret_cast<const int *>(plan.meta + clampc(c + kWarmAhead))[opaque];
                }
                if constexpr (FF) {
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct)
                        if (ct == 0 || two) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) x0[ct][t] = project(ft0[ct], dterm[ct][t], t);
                        }
                }
            }
            if (n == (NL > 2 ? 1 : 0)) {
                // the rest of the batch, behind the second layer's matrix instructions
                const bool two_next = m1.y > kTileNodes;
                m2 = load_uniform(plan.meta + clampc(c + 2));
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) {
                    if (ct > 0 && !two_next) continue;
                    const int r = 4 * ct + kg;
                    const int rr = (r < m1.y) ? r : 0;
                    ent1[ct] = *reinterpret_cast<const u32x4 *>(plan.ent + static_cast<size_t>(clampc(c + 1)) * CH +
                                                               static_cast<uint32_t>(r));
                    vg1[ct] = (order + m1.x)[static_cast<uint32_t>(rr)];
                    if constexpr (FF) {
                        ft0[ct] = *reinterpret_cast<const f32x4 *>(featb + m1.x + static_cast<uint32_t>(rr));
                    } else {
#pragma unroll
                        for (int t = 0; t < TPW; ++t) {
                            x1[ct][t] = (xb + static_cast<size_t>(m1.x) * H)[static_cast<uint32_t>(rr * H + wc0 + 16 * t + col)];
                            if constexpr (BW)
                                mk1[ct][t] = (mask4 + static_cast<size_t>(m1.x) * H)[static_cast<uint32_t>(rr * H + wc0 + 16 * t + col)];
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < PFN; ++i) {     // ids staged two chunks ahead of their data
                    const int f = (lane + 64 * i) / QW;
                    fid1[i] = (f < FCAP) ? (plan.far + static_cast<size_t>(clampc(c + 2)) * FCAP)[static_cast<uint32_t>(f)] : -1;
                }
            }

            if (n == NL - 1) {
                // Behind the last layer's matrix instructions: the reachability bits of this
                // chunk's nodes go to HBM and the far messages of the next chunk into the table.
                if constexpr (!BW) {
#pragma unroll
                    for (int ct = 0; ct < NT; ++ct) {
                        const int r = ct * kTileNodes + kg;
                        reach[static_cast<uint32_t>((wave == 0 && col == 0 && r < rows) ? vg0[ct] : sink_row)] =
                            static_cast<uint8_t>(bit0[ct]);
                    }
                }
                // Wait for this wave's prefetch batch whether or not a lane uses it: the stores
                // that preceded it are then complete too (see the note at the prefetch).
#pragma unroll
                for (int i = 0; i < PFN; ++i) asm volatile("" ::"v"(pf[i][0]), "v"(pf_reach[i]), "v"(fid1[i]));
                asm volatile("" ::"v"(warm));
                // ... and for the rest of the batch, which the next chunk then uses without waiting
#pragma unroll
                for (int ct = 0; ct < NT; ++ct) {
                    asm volatile("" ::"v"(ent1[ct][0]), "v"(vg1[ct]));
                    if constexpr (FF) {
                        asm volatile("" ::"v"(ft0[ct][0]));
                    } else {
#pragma unroll
                        for (int t = 0; t < TPW; ++t) asm volatile("" ::"v"(x1[ct][t]));
                        if constexpr (BW) {
#pragma unroll
                            for (int t = 0; t < TPW; ++t) asm volatile("" ::"v"(mk1[ct][t]));
                        }
                    }
                }
                if (has_next) {
                    // An offset the compiler cannot see through, defined only here: without it
                    // the staged LDS stores below are scheduled right behind their loads, which
                    // puts the whole HBM latency back on the critical path.
                    int late = 0;
                    asm volatile("" : "+v"(late));
#pragma unroll
                    for (int i = 0; i < PFN; ++i) {     // far messages of chunk c + 1, this wave's columns
                        if (m1.z <= i * (64 / QW)) continue;
                        const int e = lane + 64 * i;
                        const int f = e / QW, q = e - f * QW;
                        if (f < m1.z) {
                            const int slot = RING * CH + (par ^ 1) * FCAP + f;
                            const uint32_t flag = (!BW && ((pf_reach[i] != 0) | pf_cur[i])) ? 0x80000000u : 0u;
                            f32x4 v;
#pragma unroll
                            for (int k = 0; k < 4; ++k) v[k] = __uint_as_float(__float_as_uint(pf[i][k]) | flag);
                            *reinterpret_cast<f32x4 *>(msgtab + slot * LDM + wc0 + 4 * q + late) = v;
                        }
                    }
                }
            }

            epilogue(0);
            if (two) epilogue(1);

            // The table rows that chunk c + 1 sums were all written by this wave (its own
            // columns), so its gather follows without a barrier.
            if (n == NL - 1 && has_next) gather(m1.w, (m1.y + kTileNodes - 1) / kTileNodes, ent1, bit0, mk1, gs0);
            lds_barrier();
        }

        m0 = m1;
        m1 = m2;
#pragma unroll
        for (int ct = 0; ct < NT; ++ct) {
            vg0[ct] = vg1[ct];
            if constexpr (!FF) {
#pragma unroll
                for (int t = 0; t < TPW; ++t) x0[ct][t] = x1[ct][t];
            }
            if constexpr (BW) {
#pragma unroll
                for (int t = 0; t < TPW; ++t) mk0[ct][t] = mk1[ct][t];
            }
        }
    }
}

// Raw features of every node in the bucket order of both directions (Section 2.1 features;
// the device and the is-current flag travel as bits).
__global__ __launch_bounds__(256) void k_bucket_feats(GraphView gv, const float *__restrict__ feats,
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
    featb[gv.pos[0][v]] = rec;
    featb[static_cast<size_t>(gv.n_tot) + gv.pos[1][v]] = rec;
}

}  // namespace

// Packs the f and g weights of both directions into MFMA B-operand fragments.
// Index: ((((dir * 2L + n) * MT + mt) * KS + ks) * WS + ws) * 64 + lane, n = g layers then f
// layers; lane l holds W[32 ks + 8 (l / 16) + i][16 mt + l % 16], i = 0..7, as bf16 part ws
// of the exact three-way split (ws = 0 only when the weights are bf16 already).
// With `reverse`, the fragments of the reverse pass: index dir is the direction whose chunks are
// walked, the weights are those of the other direction, transposed, f's layers from the last to
// the first and then g's (biases are not used there).
void pack_sweep_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                        std::vector<float> *bias, bool reverse)
{
    const int H = mv.H, L = mv.L, MT = H / 16, KS = H / 32, NL = 2 * L;
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
                            const int k = 32 * ks + 8 * (lane / 16) + i, m = 16 * mt + lane % 16;
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
                       bool first_sweep, bool more_sweeps, float *keep, size_t keep_stride, hipStream_t s)
{
    if (gv.B == 0) return;
    // keep: where a single sweep also stores a_v and the layer outputs for the reverse pass (TR)
    const bool tr = keep && first_sweep && !more_sweeps;
    SweepParams P{gv, wfrag, bias, ws.emb, ws.xb, ws.msg, ws.reach, fa.cur_node,
                  ws.featb, first_sweep ? mv.blob + mv.proj.w : nullptr, mv.D, nullptr, tr ? keep : nullptr,
                  tr ? keep_stride : 0};
    if (first_sweep)
        hipLaunchKernelGGL(k_bucket_feats, dim3((gv.n_tot + 255) / 256), dim3(256), 0, s, gv, fa.node_feats,
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
// holds the outside gradient of every state on entry (also given in bucket order in extb) and the
// gradient of the sweep's input on return; dagg [2 n_tot + 2, H] must have its row 2 n_tot zero.
void launch_sweep_mfma_bw(const GraphView &gv, const ModelView &mv, const uint4 *wfrag, const float *bias,
                          int WS, const int32_t *cur_node, float *demb, float *extb, float *dagg,
                          const uint8_t *mask4, float *delta, size_t delta_stride, hipStream_t s)
{
    if (gv.B == 0) return;
    SweepParams P{gv, wfrag, bias, demb, extb, dagg, nullptr, cur_node, nullptr, nullptr, mv.D,
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
