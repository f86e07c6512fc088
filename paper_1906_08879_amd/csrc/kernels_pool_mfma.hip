// Matrix-core pooling kernel for gfx950: Section 2.2 step 3,
//   P[i][d] = sum over nodes u of set i placed on device d of l_i([td_u ; bu_u]),
// for H in {32, 64, 128} and one or two layers in l_i.
//
// One workgroup per (graph, slice of its nodes, set).  It scans its nodes in node order, queues
// the nodes of its set, and pushes them through l_i sixteen at a time:
//   * the fp32 embedding row of a node is split exactly into three bf16 parts (truncation);
//     the hi, mid and lo parts of the sixteen nodes form three 16-row MFMA A tiles, so a lane
//     finds the three partial products of (node, column) in the same element of three
//     accumulators and adds them there: no cross-lane traffic and no wasted rows;
//   * the weights of l_i are the B operand and stay in registers for the whole kernel;
//   * the rows of the next batch are loaded from HBM while the current one is computed;
//   * the per-device sums are taken in registers, by the lane that holds a node's output in
//     its accumulators, in batch order; the four lanes of a column are added once at the end
//     in a fixed order, so the result is bitwise reproducible.
#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kThreads = 256;
constexpr int kBatch = 16;          // nodes per batch: one MFMA row tile per bf16 part
constexpr int kWindow = 256;        // nodes classified per scan step
constexpr int kQueue = 512;         // circular queue of node ids (power of two > kWindow + kBatch)

__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

__device__ __forceinline__ uint32_t pack_hi16(float lo_word, float hi_word)
{
    return __builtin_amdgcn_perm(__float_as_uint(hi_word), __float_as_uint(lo_word), 0x07060302u);
}

__device__ __forceinline__ float trunc_bf16(float x)
{
    return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u);
}

struct PoolParams {
    GraphView gv;
    const uint4 *wfrag;        // packed B fragments of l_par, l_chi, l_pll (see pack_pool_weights)
    const float *bias;         // [3 sets][L][H]
    const float *emb;          // [n_tot, 2H]
    const uint8_t *reach;      // [2, n_tot]
    const int32_t *placement;  // [n_tot]
    const int32_t *cur_node;   // [B]
    float *partial;            // [B, max_slices, 3, G, H] sums over a slice of the graph's nodes
    int max_slices;
    int D, G;
    float *keep;               // (KEEP) [L][n_tot, H]: the outputs of l's layers for every node of a set
    int single;                // 1: every node other than v* belongs to the first set
};

// KEEP: the outputs of every layer of l_i are also written to HBM, by the lane that holds them,
// for the reverse pass (a node belongs to one set and is handled by one workgroup).
template <int H, int WS, int L, bool KEEP = false>
__global__ __launch_bounds__(kThreads, 2) void k_pool_mfma(PoolParams P)
{
    constexpr int K1 = 2 * H;                    // input width of the first layer
    constexpr int KS1 = K1 / 32, KS2 = H / 32;
    constexpr int NTL = H / 16;                  // output column tiles
    constexpr int TPW = (NTL + 3) / 4;           // column tiles per wave
    constexpr int LD1 = K1 + 8, LD2 = H + 8;     // bf16 row strides
    constexpr int QPR = K1 / 4;                  // float4 per embedding row
    constexpr int NLD = kBatch * QPR / kThreads; // float4 loads per thread and batch
    static_assert(kBatch * QPR % kThreads == 0, "batch rows must divide over the threads");

    // [part][node][k] bf16 parts of the input rows and of the layer-1 outputs; the same memory
    // holds the final cross-lane reduction
    constexpr size_t kAct1 = sizeof(__bf16) * 3 * kBatch * LD1, kAct2 = sizeof(__bf16) * 3 * kBatch * LD2;
    constexpr size_t kRed = sizeof(float) * 4 * kMaxD * H;
    __shared__ __attribute__((aligned(16))) unsigned char smem[kAct1 + kAct2 > kRed ? kAct1 + kAct2 : kRed];
    __bf16 (*act1)[kBatch][LD1] = reinterpret_cast<__bf16 (*)[kBatch][LD1]>(smem);
    __bf16 (*act2)[kBatch][LD2] = reinterpret_cast<__bf16 (*)[kBatch][LD2]>(smem + kAct1);
    __shared__ int queue[kQueue];
    __shared__ int batch_node[2][kBatch];
    __shared__ int batch_dev[2][kBatch];
    __shared__ int wave_cnt[4];

    const int set = blockIdx.x, slice = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const GraphView &gv = P.gv;
    const int g0 = gv.node_off[b], g_n = gv.node_off[b + 1] - g0;
    const int cl = P.cur_node[b];
    const int cur = (cl >= 0 && cl < g_n) ? g0 + cl : -1;
    const int G = P.G, D = P.D;
    // the graph's nodes are cut into slices (same rule as the generic pooling kernel); this
    // workgroup owns nodes [n0, n0 + n_b)
    int slices = (g_n + kPoolChunk - 1) / kPoolChunk;
    if (slices > P.max_slices) slices = P.max_slices;
    if (slice >= slices) return;
    const int per = (g_n + slices - 1) / slices;
    const int n0 = g0 + slice * per;
    const int n_b = min(per, g_n - slice * per);

    // ---- weights of l_set into registers (B operand: lane holds column 16 nt + col)
    bf16x8 W1[TPW][KS1][WS];
    bf16x8 W2[L > 1 ? TPW : 1][L > 1 ? KS2 : 1][WS];
    float bias1[TPW], bias2[TPW];
    {
        const size_t per_set = static_cast<size_t>(NTL) * (KS1 + (L > 1 ? KS2 : 0)) * WS * 64;
        const uint4 *base = P.wfrag + set * per_set;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            const int nt = wave * TPW + t;
            const int ntc = nt < NTL ? nt : NTL - 1;
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
                for (int ws = 0; ws < WS; ++ws) {
                    const uint4 raw = base[((static_cast<size_t>(ntc) * KS1 + ks) * WS + ws) * 64 + lane];
                    W1[t][ks][ws] = *reinterpret_cast<const bf16x8 *>(&raw);
                }
            bias1[t] = P.bias[(set * L + 0) * H + ntc * 16 + col];
            bias2[t] = 0.0f;
            if constexpr (L > 1) {
                const uint4 *base2 = base + static_cast<size_t>(NTL) * KS1 * WS * 64;
#pragma unroll
                for (int ks = 0; ks < KS2; ++ks)
#pragma unroll
                    for (int ws = 0; ws < WS; ++ws) {
                        const uint4 raw = base2[((static_cast<size_t>(ntc) * KS2 + ks) * WS + ws) * 64 + lane];
                        W2[t][ks][ws] = *reinterpret_cast<const bf16x8 *>(&raw);
                    }
                bias2[t] = P.bias[(set * L + 1) * H + ntc * 16 + col];
            }
        }
    }
    for (int i = tid; i < static_cast<int>((kAct1 + kAct2) / 4); i += kThreads) reinterpret_cast<uint32_t *>(smem)[i] = 0u;
    __syncthreads();

    int q_head = 0;           // position of the oldest queued node (uniform)
    int q_len = 0;            // queued nodes not yet batched (uniform)
    int scan = 0;             // next node of the graph to classify (uniform)
    int have = 0;             // nodes of the batch whose rows are in flight (uniform)
    int slot = 0;             // batch_node buffer of the in-flight batch
    f32x4 x[NLD];             // the in-flight rows: item e = tid + i * 256 -> (node e / QPR, float4 e % QPR)
    float acc_dev[kMaxD][TPW];   // per-device sums over this lane's nodes (4 kg .. 4 kg + 3 of every batch) and columns
#pragma unroll
    for (int d = 0; d < kMaxD; ++d)
#pragma unroll
        for (int t = 0; t < TPW; ++t) acc_dev[d][t] = 0.0f;

    // Fills the queue until it holds a full batch or the graph is exhausted.
    auto refill = [&]() {
        while (q_len < kBatch && scan < n_b) {
            const int v = n0 + scan + tid;
            bool mine = false;
            if (scan + tid < n_b && v != cur) {
                const int c = P.single ? 0 : (P.reach[static_cast<size_t>(gv.n_tot) + v] ? 0 : (P.reach[v] ? 1 : 2));
                mine = (c == set);
            }
            const unsigned long long m = __ballot(mine);
            if (lane == 0) wave_cnt[wave] = __popcll(m);
            lds_barrier();
            int base = q_len;
            for (int w = 0; w < wave; ++w) base += wave_cnt[w];
            if (mine) queue[(q_head + base + __popcll(m & ((1ull << lane) - 1ull))) & (kQueue - 1)] = v;
            q_len += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
            scan += kWindow;
            lds_barrier();
        }
    };
    // Takes up to a batch from the queue and issues the loads of its rows.
    auto issue = [&]() {
        have = q_len < kBatch ? q_len : kBatch;
        slot ^= 1;
        if (tid < kBatch) batch_node[slot][tid] = tid < have ? queue[(q_head + tid) & (kQueue - 1)] : -1;
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = tid + i * kThreads;
            const int node = e / QPR, q = e - node * QPR;
            const int v = node < have ? queue[(q_head + node) & (kQueue - 1)] : n0;   // any valid row if empty
            x[i] = *reinterpret_cast<const f32x4 *>(P.emb + static_cast<size_t>(v) * K1 + 4 * q);
        }
        q_head = (q_head + have) & (kQueue - 1);
        q_len -= have;
        lds_barrier();      // orders LDS only: the row loads stay in flight
    };

    refill();
    issue();
    while (have > 0) {
        const int cnt = have;
        const int my_slot = slot;
        // ---- (1) split the rows that arrived and publish them as MFMA A rows
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = tid + i * kThreads;
            const int node = e / QPR, q = e - node * QPR;
            float r[4], l[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                r[k] = x[i][k] - trunc_bf16(x[i][k]);
                l[k] = r[k] - trunc_bf16(r[k]);
            }
            *reinterpret_cast<uint2 *>(&act1[0][node][4 * q]) = uint2{pack_hi16(x[i][0], x[i][1]), pack_hi16(x[i][2], x[i][3])};
            *reinterpret_cast<uint2 *>(&act1[1][node][4 * q]) = uint2{pack_hi16(r[0], r[1]), pack_hi16(r[2], r[3])};
            *reinterpret_cast<uint2 *>(&act1[2][node][4 * q]) = uint2{pack_hi16(l[0], l[1]), pack_hi16(l[2], l[3])};
        }
        if (tid < kBatch) {
            const int v = batch_node[my_slot][tid];
            int dev = -1;
            if (v >= 0) {
                const int d = P.placement[v];
                dev = (d >= 0 && d < D) ? (G == 1 ? 0 : d) : -1;
            }
            batch_dev[my_slot][tid] = dev;
        }
        // ---- (2) next batch: queue it and put its loads in flight
        refill();
        issue();          // ends with a barrier: act1 and batch_dev are visible

        // ---- (3) layer 1.  acc[part][t]: element i of lane (col, kg) belongs to node 4 kg + i
        // and output column 16 nt + col.  3 * TPW independent accumulation chains are in
        // flight, which hides the latency of a dependent MFMA.  Rows past the batch's end hold
        // stale data that is never summed.
        f32x4 acc[3][TPW];
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int t = 0; t < TPW; ++t) acc[p][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS1; ++ks)
#pragma unroll
            for (int p = 0; p < 3; ++p) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&act1[p][col][32 * ks + 8 * kg]);
#pragma unroll
                for (int t = 0; t < TPW; ++t)
#pragma unroll
                    for (int ws = 0; ws < WS; ++ws)
                        acc[p][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, W1[t][ks][ws], acc[p][t], 0, 0, 0);
            }
        if constexpr (L > 1) {
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int nt = wave * TPW + t;
                if (nt >= NTL) continue;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float y = fmaxf(acc[0][t][i] + acc[1][t][i] + acc[2][t][i] + bias1[t], 0.0f);
                    const float r = y - trunc_bf16(y);
                    const float l = r - trunc_bf16(r);
                    const int node = 4 * kg + i, c = 16 * nt + col;
                    if constexpr (KEEP) {
                        if (node < cnt) P.keep[static_cast<size_t>(batch_node[my_slot][node]) * H + c] = y;
                    }
                    reinterpret_cast<unsigned short *>(&act2[0][node][c])[0] = static_cast<unsigned short>(__float_as_uint(y) >> 16);
                    reinterpret_cast<unsigned short *>(&act2[1][node][c])[0] = static_cast<unsigned short>(__float_as_uint(r) >> 16);
                    reinterpret_cast<unsigned short *>(&act2[2][node][c])[0] = static_cast<unsigned short>(__float_as_uint(l) >> 16);
                }
            }
            lds_barrier();
            // ---- (4) layer 2
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int t = 0; t < TPW; ++t) acc[p][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS2; ++ks)
#pragma unroll
                for (int p = 0; p < 3; ++p) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(&act2[p][col][32 * ks + 8 * kg]);
#pragma unroll
                    for (int t = 0; t < TPW; ++t)
#pragma unroll
                        for (int ws = 0; ws < WS; ++ws)
                            acc[p][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, W2[t][ks][ws], acc[p][t], 0, 0, 0);
                }
        }
        // ---- (5) per-device sums in registers: lane (col, kg) adds the outputs of its own
        // nodes (4 kg + i) to the sum of the node's device; nodes past the end of the batch
        // have device -1 and are never added
        float y[4][TPW];
        int dv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int node = 4 * kg + i;
            dv[i] = node < cnt ? batch_dev[my_slot][node] : -1;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const float bl = (L > 1) ? bias2[t] : bias1[t];
                y[i][t] = fmaxf(acc[0][t][i] + acc[1][t][i] + acc[2][t][i] + bl, 0.0f);
                if constexpr (KEEP) {
                    const int nt = wave * TPW + t;
                    if (node < cnt && nt < NTL)
                        P.keep[(static_cast<size_t>(L - 1) * gv.n_tot + batch_node[my_slot][node]) * H + 16 * nt + col] = y[i][t];
                }
            }
        }
        // rows past the end of the batch hold earlier, finite outputs: weight 0 removes them
#pragma unroll
        for (int d = 0; d < kMaxD; ++d) {
            if (d >= G) break;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float wgt = dv[i] == d ? 1.0f : 0.0f;
#pragma unroll
                for (int t = 0; t < TPW; ++t) acc_dev[d][t] = fmaf(wgt, y[i][t], acc_dev[d][t]);
            }
        }
    }

    // ---- the four lanes of a column (kg = 0..3) are added in order; the buffer of the first
    // layer's A rows is free now and holds the partial sums
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);             // [4 kg][G][H]
#pragma unroll
    for (int t = 0; t < TPW; ++t) {
        const int nt = wave * TPW + t;
        if (nt >= NTL) continue;
#pragma unroll
        for (int d = 0; d < kMaxD; ++d) {
            if (d >= G) break;
            red[(kg * G + d) * H + 16 * nt + col] = acc_dev[d][t];
        }
    }
    __syncthreads();
    float *dst = P.partial + (((static_cast<size_t>(b) * P.max_slices + slice) * 3 + set) * G) * H;
    for (int i = tid; i < G * H; i += kThreads)
        dst[i] = ((red[i] + red[G * H + i]) + red[2 * G * H + i]) + red[3 * G * H + i];
}

// Appends the MFMA B-operand fragments of one layer: index ((nt * KS + ks) * WS + ws) * 64 + lane,
// lane l holds W[32 ks + 8 (l / 16) + i][16 nt + l % 16], i = 0..7, as bf16 part ws of the exact
// three-way split of the weight (ws = 0 only when the weights are bf16 already).
void append_fragments(const float *blob, const LayerRef &lr, int WS, std::vector<uint16_t> *out)
{
    const int NTL = lr.n_out / 16, KS = lr.n_in / 32;
    const size_t base = out->size();
    out->resize(base + static_cast<size_t>(NTL) * KS * WS * 64 * 8, 0);
    auto to_bf16 = [](float x) {
        uint32_t u;
        std::memcpy(&u, &x, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return static_cast<uint16_t>(u >> 16);
    };
    auto from_bf16 = [](uint16_t h) {
        const uint32_t u = static_cast<uint32_t>(h) << 16;
        float x;
        std::memcpy(&x, &u, 4);
        return x;
    };
    for (int nt = 0; nt < NTL; ++nt)
        for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int i = 0; i < 8; ++i) {
                    const int k = 32 * ks + 8 * (lane / 16) + i, m = 16 * nt + lane % 16;
                    float rest = blob[lr.w + static_cast<size_t>(k) * lr.n_out + m];
                    for (int ws = 0; ws < WS; ++ws) {
                        const uint16_t part = to_bf16(rest);
                        rest -= from_bf16(part);
                        (*out)[base + ((((static_cast<size_t>(nt) * KS + ks) * WS + ws) * 64 + lane) * 8) + i] = part;
                    }
                }
}

}  // namespace

void pack_pool_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                       std::vector<float> *bias)
{
    frag->clear();
    bias->assign(static_cast<size_t>(3) * mv.L * mv.H, 0.0f);
    for (int set = 0; set < 3; ++set)
        for (int l = 0; l < mv.L; ++l) {
            append_fragments(blob, mv.l[set].layer[l], WS, frag);
            for (int h = 0; h < mv.H; ++h)
                (*bias)[(static_cast<size_t>(set) * mv.L + l) * mv.H + h] = blob[mv.l[set].layer[l].b + h];
        }
}

bool pool_mfma_supported(int H, int L, int weight_dtype)
{
    if (L < 1 || L > 2) return false;
    if (weight_dtype == PL_WEIGHTS_BF16) return H == 32 || H == 64 || H == 128;
    return H == 32 || H == 64;
}

void launch_pool_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                      const ForwardArgs &fa, const uint4 *wfrag, const float *bias, int WS,
                      float *keep, hipStream_t s)
{
    if (gv.B == 0) return;
    PoolParams P{gv, wfrag, bias, ws.emb, ws.reach, fa.placement, fa.cur_node, ws.partial,
                 kPoolSlices, mv.D, mv.G, keep, mv.single_set};
    const dim3 grid(3, kPoolSlices, gv.B), block(kThreads);
#define PL_CASE(HH, WW, LL)                                                          \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                      \
        if (keep)                                                                    \
            hipLaunchKernelGGL((k_pool_mfma<HH, WW, LL, true>), grid, block, 0, s, P); \
        else                                                                         \
            hipLaunchKernelGGL((k_pool_mfma<HH, WW, LL>), grid, block, 0, s, P);     \
        return;                                                                      \
    }
    PL_CASE(128, 1, 2) PL_CASE(128, 1, 1)
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
}

}  // namespace pl
