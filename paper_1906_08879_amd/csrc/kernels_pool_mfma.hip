// Matrix-core pooling for gfx950: Section 2.2 step 3,
//   P[i][d] = sum over nodes u of set i placed on device d of l_i([td_u ; bu_u]),
// for H in {32, 64, 128} and one or two layers in l_i.
//
// Two kernels per pass:
//   k_pool_sort   one workgroup per graph: a counting sort of the graph's nodes by
//                 key = (set, device group), without atomics (a thread counts and places a
//                 contiguous block of nodes), so the order is the same on every run;
//   k_pool_stream (H = 128, bf16 weights) one workgroup per graph, or per (set, graph) in small
//                 batches; every wave walks tiles of its own with the weights in LDS, the rows
//                 coming straight from HBM and the two layers chained in registers (see there);
//   k_pool_tiles  (H <= 64) one workgroup per (set, slice of the set's tiles, graph).  A tile is
//                 up to sixteen nodes of ONE key, so the sum over a tile's rows needs no per-device
//                 selection: a lane adds its four nodes' outputs to one running sum, which is
//                 written out when the device changes.
// In k_pool_tiles:
//   * the fp32 embedding row of a node is split exactly into three bf16 parts (truncation);
//     the hi, mid and lo parts of the sixteen nodes form three 16-row MFMA A tiles, so a lane
//     finds the three partial products of (node, column) in the same element of three
//     accumulators and adds them there: no cross-lane traffic and no wasted rows;
//   * the weights of l_i are the B operand and stay in registers for the whole kernel;
//   * the rows of the next tile are loaded from HBM while the current one is computed;
//   * a lane that owns two output columns hands them to the second layer as one word per part
//     (the second layer's contraction index is permuted to match, see pack_pool_weights);
//   * all sums are taken in a fixed order, so the result is bitwise reproducible.
#include <type_traits>

#include "internal.h"

namespace pl {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

constexpr int kThreads = 256;
constexpr int kBatch = 16;          // nodes per tile: one MFMA row tile per bf16 part
constexpr int kMaxKeys = 3 * kMaxD; // (set, device group) keys of a graph
constexpr int kAhead = 2;            // k-steps between reading an A fragment from LDS and using it

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

// ---- counting sort of a graph's nodes by (set, device group).  klist gets the graph's node ids
// (global) grouped by key, koff[b][k] the position (within the graph) of key k's first node,
// koff[b][3G] the number of pooled nodes.  The current node and nodes with a device id outside
// [0, D) belong to no key.  Thread t counts, then places, the nodes of its own contiguous block.
__global__ __launch_bounds__(kThreads) void k_pool_sort(GraphView gv, const uint8_t *__restrict__ reach,
                                                        const int32_t *__restrict__ placement,
                                                        const int32_t *__restrict__ cur_node, int D, int G,
                                                        int single, int32_t *__restrict__ klist,
                                                        int32_t *__restrict__ koff)
{
    __shared__ uint16_t hist[kMaxKeys][kThreads];    // nodes of key k in thread t's block, then their first position
    __shared__ int total[kMaxKeys + 1];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const int K = 3 * G;
    const int per = (n_b + kThreads - 1) / kThreads;
    const int lo = n0 + min(tid * per, n_b), hi = n0 + min((tid + 1) * per, n_b);
    auto key_of = [&](int v) {
        if (v == cur) return -1;
        const int d = placement[v];
        if (d < 0 || d >= D) return -1;
        const int set = single ? 0 : (reach[static_cast<size_t>(gv.n_tot) + v] ? 0 : (reach[v] ? 1 : 2));
        return set * G + (G == 1 ? 0 : d);
    };
    for (int k = 0; k < K; ++k) hist[k][tid] = 0;
    // The keys of a thread's nodes are formed sixteen at a time, all their loads in flight together;
    // the first sixteen stay in registers for the placing pass.
    constexpr int KB = 16;
    int first_keys[KB];
#pragma unroll
    for (int u = 0; u < KB; ++u) first_keys[u] = lo + u < hi ? key_of(lo + u) : -1;
#pragma unroll
    for (int u = 0; u < KB; ++u)
        if (first_keys[u] >= 0) hist[first_keys[u]][tid] += 1;
    for (int base = lo + KB; base < hi; base += KB) {
        int keys[KB];
#pragma unroll
        for (int u = 0; u < KB; ++u) keys[u] = base + u < hi ? key_of(base + u) : -1;
#pragma unroll
        for (int u = 0; u < KB; ++u)
            if (keys[u] >= 0) hist[keys[u]][tid] += 1;
    }
    __syncthreads();
    if (tid < K) {                                   // exclusive prefix over the threads, per key
        int run = 0;
        for (int t = 0; t < kThreads; ++t) {
            const int c = hist[tid][t];
            hist[tid][t] = static_cast<uint16_t>(run);
            run += c;
        }
        total[tid] = run;
    }
    __syncthreads();
    if (tid == 0) {                                  // exclusive prefix over the keys
        int run = 0;
        for (int k = 0; k < K; ++k) {
            const int c = total[k];
            total[k] = run;
            run += c;
        }
        total[K] = run;
    }
    __syncthreads();
    int32_t *kb = koff + static_cast<size_t>(b) * (kMaxKeys + 1);
    if (tid <= K) kb[tid] = total[tid];
    auto place = [&](int v, int k) {
        if (k < 0) return;
        const int at = total[k] + hist[k][tid];
        hist[k][tid] += 1;
        klist[n0 + at] = v;
    };
#pragma unroll
    for (int u = 0; u < KB; ++u) place(lo + u, first_keys[u]);
    for (int base = lo + KB; base < hi; base += KB) {
        int keys[KB];
#pragma unroll
        for (int u = 0; u < KB; ++u) keys[u] = base + u < hi ? key_of(base + u) : -1;
#pragma unroll
        for (int u = 0; u < KB; ++u) place(base + u, keys[u]);
    }
}

struct PoolParams {
    GraphView gv;
    const uint4 *wfrag;        // packed B fragments of l_par, l_chi, l_pll (see pack_pool_weights)
    const float *bias;         // [3 sets][L][H]
    const float *emb;          // [n_tot, 2H]
    const int32_t *klist;      // [n_tot] node ids grouped by key, per graph
    const int32_t *koff;       // [B][kMaxKeys + 1]
    float *partial;            // [B, max_slices, 3, G, H] sums over a slice of the set's tiles
    int max_slices;
    int G;
    float *keep;               // (KEEP) [L][n_tot, H]: the outputs of l's layers for every node of a set
};

// KEEP: the outputs of every layer of l_i are also written to HBM, by the lane that holds them,
// for the reverse pass (a node belongs to one set and is handled by one workgroup).
template <int H, int WS, int L, bool KEEP = false>
__global__ __launch_bounds__(kThreads, 2) void k_pool_tiles(PoolParams P)
{
    constexpr int K1 = 2 * H;                    // input width of the first layer
    constexpr int KS1 = K1 / 32, KS2 = H / 32;
    constexpr int NTL = H / 16;                  // output column tiles
    constexpr int TPW = (NTL + 3) / 4;           // column tiles per wave
    // bf16 row strides: K / 2 + 8 words.  Measured on this chip (SQ_LDS_BANK_CONFLICT): a
    // ds_read_b128 of A rows then runs at its full rate of four cycles (K / 2 + 4 words: eight).
    constexpr int LD1 = K1 + 16, LD2 = H + 16;
    constexpr int QPR = K1 / 4;                  // float4 per embedding row
    constexpr int NLD = kBatch * QPR / kThreads; // float4 loads per thread and tile
    static_assert(kBatch * QPR % kThreads == 0, "tile rows must divide over the threads");
    static_assert(TPW == 1 || TPW == 2, "a lane owns one or two output columns");

    // [part][node][k] bf16 parts of the input rows and of the layer-1 outputs
    __shared__ __attribute__((aligned(16))) __bf16 act1[2][3][kBatch][LD1];   // two tiles: one is read while the next is written
    __shared__ __attribute__((aligned(16))) __bf16 act2[L > 1 ? 3 : 1][kBatch * LD2];
    auto act2_at = [&](int part, int node, int k) __attribute__((always_inline)) {
        return &act2[part][node * LD2 + k];
    };
    __shared__ int tile_node[8][kBatch];     // node ids of the tiles t - 1 .. t + 4 (slot = tile & 7)

    const int set = blockIdx.x, slice = blockIdx.y, b = blockIdx.z;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const GraphView &gv = P.gv;
    const int g0 = gv.node_off[b], g_n = gv.node_off[b + 1] - g0;
    const int G = P.G;
    // a graph's sets are cut into slices (as many as the generic pooling kernel uses chunks)
    int slices = (g_n + kPoolChunk - 1) / kPoolChunk;
    if (slices > P.max_slices) slices = P.max_slices;
    if (slice >= slices) return;
    // tiles of this set: for every device group ceil(count / 16), in device order; this
    // workgroup takes the tiles [t_lo, t_hi) of that list
    const int32_t *kb = P.koff + static_cast<size_t>(b) * (kMaxKeys + 1) + set * G;
    int n_tiles = 0;
    for (int d = 0; d < G; ++d) n_tiles += (kb[d + 1] - kb[d] + kBatch - 1) / kBatch;
    const int t_lo = static_cast<int>(static_cast<long long>(n_tiles) * slice / slices);
    const int t_hi = static_cast<int>(static_cast<long long>(n_tiles) * (slice + 1) / slices);
    float *dst = P.partial + (((static_cast<size_t>(b) * P.max_slices + slice) * 3 + set) * G) * H;
    if (t_lo >= t_hi) {
        for (int i = tid; i < G * H; i += kThreads) dst[i] = 0.0f;
        return;
    }

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
    const bool my_cols = wave * TPW < NTL;        // narrow networks leave the last waves without columns

    // ---- tile walk: (device group d, first node position p, node count) of tile t
    int d_cur = 0, d_first = 0;                   // device group of the walk; tiles before it
    auto seek = [&](int t) {                      // t only grows
        while (d_cur < G && t >= d_first + (kb[d_cur + 1] - kb[d_cur] + kBatch - 1) / kBatch) {
            d_first += (kb[d_cur + 1] - kb[d_cur] + kBatch - 1) / kBatch;
            ++d_cur;
        }
    };
    // Rows travel two tiles ahead of the matrix instructions (a workgroup keeps 32 KB of loads
    // in flight); the node ids of a tile are staged in LDS earlier still, so a row load never
    // waits for an id load.  Ring of eight id slots (slot = tile & 7).
    // The id of a tile's node tid (threads 0..15) is fetched before the row loads of the same
    // iteration are issued and published after them: loads return in order, so the wait for the
    // id then leaves the row loads in flight.
    auto fetch_id = [&](int t, int &cnt, int &dev) {
        seek(t);
        const int p = kb[d_cur] + (t - d_first) * kBatch;
        cnt = min(kBatch, kb[d_cur + 1] - p);
        dev = d_cur;
        return tid < kBatch ? P.klist[g0 + p + (tid < cnt ? tid : 0)] : 0;   // rows past the end repeat the first
    };
    auto publish_id = [&](int t, int id) {
        if (tid < kBatch) tile_node[t & 7][tid] = id;
    };
    auto load_rows = [&](int t, f32x4 (&x)[NLD]) {
#pragma unroll
        for (int i = 0; i < NLD; ++i) {
            const int e = tid + i * kThreads;
            const int node = e / QPR, q = e - node * QPR;
            x[i] = *reinterpret_cast<const f32x4 *>(P.emb + static_cast<size_t>(tile_node[t & 7][node]) * K1 + 4 * q);
        }
    };
    // Splits item i of a tile's rows exactly into three bf16 parts and writes them as MFMA A rows.
    auto split_item = [&](int buf, const f32x4 (&x)[NLD], int i) {
        const int e = tid + i * kThreads;
        const int node = e / QPR, q = e - node * QPR;
        float r[4], l[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            r[k] = x[i][k] - trunc_bf16(x[i][k]);
            l[k] = r[k] - trunc_bf16(r[k]);
        }
        *reinterpret_cast<uint2 *>(&act1[buf][0][node][4 * q]) = uint2{pack_hi16(x[i][0], x[i][1]), pack_hi16(x[i][2], x[i][3])};
        *reinterpret_cast<uint2 *>(&act1[buf][1][node][4 * q]) = uint2{pack_hi16(r[0], r[1]), pack_hi16(r[2], r[3])};
        *reinterpret_cast<uint2 *>(&act1[buf][2][node][4 * q]) = uint2{pack_hi16(l[0], l[1]), pack_hi16(l[2], l[3])};
    };

    float run[TPW];           // running sum over this lane's nodes (4 kg .. 4 kg + 3 of every tile) of the current device group
#pragma unroll
    for (int t = 0; t < TPW; ++t) run[t] = 0.0f;
    int run_dev = -1;
    unsigned written = 0;     // device groups whose sum has been written
    // Adds the four lanes of a column (kg = 0..3) in a fixed order and writes the device group's sum.
    auto flush = [&]() {
        if (run_dev < 0) return;
#pragma unroll
        for (int t = 0; t < TPW; ++t) {
            float s = run[t];
            s += __shfl_xor(s, 16);
            s += __shfl_xor(s, 32);
            const int nt = wave * TPW + t;
            if (kg == 0 && nt < NTL) dst[run_dev * H + 16 * nt + col] = s;
            run[t] = 0.0f;
        }
        written |= 1u << run_dev;
    };

    f32x4 xa[NLD], xb[NLD];            // rows of the next two tiles, alternately
    int cnt_r[5], dev_r[5];            // nodes and device group of the tiles t .. t + 4 (uniform)
#pragma unroll
    for (int j = 0; j < 5; ++j) cnt_r[j] = dev_r[j] = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        if (t_lo + j < t_hi) publish_id(t_lo + j, fetch_id(t_lo + j, cnt_r[j], dev_r[j]));
    __syncthreads();
    load_rows(t_lo, xa);
    if (t_lo + 1 < t_hi) load_rows(t_lo + 1, xb);
#pragma unroll
    for (int i = 0; i < NLD; ++i) split_item(0, xa, i);
    if (t_lo + 2 < t_hi) load_rows(t_lo + 2, xa);

    // One tile: the matrix instructions of tile t, with the split of tile t + 1's rows (xs)
    // interleaved between the k-steps of the first layer, into the other half of act1.
    auto step = [&](int t, f32x4 (&xs)[NLD]) {
        const int cnt = cnt_r[0], dev = dev_r[0], my_slot = t & 7, buf = (t - t_lo) & 1;
        const bool more = t + 1 < t_hi;
        int id4 = 0;
        if (t + 4 < t_hi) id4 = fetch_id(t + 4, cnt_r[4], dev_r[4]);
        // every wave has finished tile t - 1 (its reads of act2 and of the other half of act1),
        // and the rows of tile t, split during tile t - 1, are visible
        lds_barrier();
        if (t + 4 < t_hi) publish_id(t + 4, id4);
        if (dev != run_dev) {
            flush();
            run_dev = dev;
        }
        // ---- layer 1.  acc[part][tt]: element i of lane (col, kg) belongs to node 4 kg + i and
        // output column 16 nt + col.  3 * TPW independent accumulation chains are in flight.
        // Rows past the tile's end hold a copy of its first row and are never summed.
        f32x4 acc[3][TPW];
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) acc[p][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
        {
            // The A fragments are read kAhead k-steps before the matrix instructions that use
            // them; the scheduling barriers keep the order written here: reads, then the matrix
            // instructions of a k-step, then a piece of the next tile's split, which the vector
            // unit works off while the matrix core is busy.
            bf16x8 a[kAhead + 1][3];
            if (my_cols) {
#pragma unroll
                for (int ks = 0; ks < kAhead && ks < KS1; ++ks)
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        a[ks][p] = *reinterpret_cast<const bf16x8 *>(&act1[buf][p][col][32 * ks + 8 * kg]);
            }
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                if (my_cols) {
                    if (ks + kAhead < KS1) {
#pragma unroll
                        for (int p = 0; p < 3; ++p)
                            a[(ks + kAhead) % (kAhead + 1)][p] =
                                *reinterpret_cast<const bf16x8 *>(&act1[buf][p][col][32 * (ks + kAhead) + 8 * kg]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int p = 0; p < 3; ++p)
#pragma unroll
                        for (int tt = 0; tt < TPW; ++tt)
#pragma unroll
                            for (int ws = 0; ws < WS; ++ws)
                                acc[p][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks % (kAhead + 1)][p], W1[tt][ks][ws],
                                                                                    acc[p][tt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                // NLD items of the split spread over the KS1 k-steps
                if (more) {
#pragma unroll
                    for (int i = 0; i < NLD; ++i)
                        if (i * KS1 / NLD == ks) split_item(buf ^ 1, xs, i);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the registers of the split rows are free: the rows of tile t + 3 go in flight
        if (t + 3 < t_hi) load_rows(t + 3, xs);
        if constexpr (L > 1) {
            if (my_cols) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int node = 4 * kg + i;
                    float y[TPW], r[TPW], l[TPW];
#pragma unroll
                    for (int tt = 0; tt < TPW; ++tt) {
                        y[tt] = fmaxf(acc[0][tt][i] + acc[1][tt][i] + acc[2][tt][i] + bias1[tt], 0.0f);
                        r[tt] = y[tt] - trunc_bf16(y[tt]);
                        l[tt] = r[tt] - trunc_bf16(r[tt]);
                        if constexpr (KEEP) {
                            if (node < cnt)
                                P.keep[static_cast<size_t>(tile_node[my_slot][node]) * H + 16 * (wave * TPW + tt) + col] = y[tt];
                        }
                    }
                    if constexpr (TPW == 2) {
                        // word 16 wave + col of a row: columns 32 wave + col and 32 wave + 16 + col
                        reinterpret_cast<uint32_t *>(act2_at(0, node, 0))[16 * wave + col] = pack_hi16(y[0], y[1]);
                        reinterpret_cast<uint32_t *>(act2_at(1, node, 0))[16 * wave + col] = pack_hi16(r[0], r[1]);
                        reinterpret_cast<uint32_t *>(act2_at(2, node, 0))[16 * wave + col] = pack_hi16(l[0], l[1]);
                    } else {
                        const int c = 16 * wave + col;
                        reinterpret_cast<unsigned short *>(act2_at(0, node, c))[0] = static_cast<unsigned short>(__float_as_uint(y[0]) >> 16);
                        reinterpret_cast<unsigned short *>(act2_at(1, node, c))[0] = static_cast<unsigned short>(__float_as_uint(r[0]) >> 16);
                        reinterpret_cast<unsigned short *>(act2_at(2, node, c))[0] = static_cast<unsigned short>(__float_as_uint(l[0]) >> 16);
                    }
                }
            }
            lds_barrier();
            // ---- layer 2
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int tt = 0; tt < TPW; ++tt) acc[p][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (my_cols) {
                bf16x8 a[kAhead + 1][3];
#pragma unroll
                for (int ks = 0; ks < kAhead && ks < KS2; ++ks)
#pragma unroll
                    for (int p = 0; p < 3; ++p) a[ks][p] = *reinterpret_cast<const bf16x8 *>(act2_at(p, col, 32 * ks + 8 * kg));
#pragma unroll
                for (int ks = 0; ks < KS2; ++ks) {
                    if (ks + kAhead < KS2) {
#pragma unroll
                        for (int p = 0; p < 3; ++p)
                            a[(ks + kAhead) % (kAhead + 1)][p] =
                                *reinterpret_cast<const bf16x8 *>(act2_at(p, col, 32 * (ks + kAhead) + 8 * kg));
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int p = 0; p < 3; ++p)
#pragma unroll
                        for (int tt = 0; tt < TPW; ++tt)
#pragma unroll
                            for (int ws = 0; ws < WS; ++ws)
                                acc[p][tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks % (kAhead + 1)][p], W2[tt][ks][ws],
                                                                                    acc[p][tt], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        // ---- the tile's rows all belong to one device group: a lane adds the outputs of its own
        // nodes (4 kg + i, those inside the tile) to the running sum, in node order
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int node = 4 * kg + i;
#pragma unroll
            for (int tt = 0; tt < TPW; ++tt) {
                const float bl = (L > 1) ? bias2[tt] : bias1[tt];
                const float y = fmaxf(acc[0][tt][i] + acc[1][tt][i] + acc[2][tt][i] + bl, 0.0f);
                if constexpr (KEEP) {
                    const int nt = wave * TPW + tt;
                    if (node < cnt && nt < NTL)
                        P.keep[(static_cast<size_t>(L - 1) * gv.n_tot + tile_node[my_slot][node]) * H + 16 * nt + col] = y;
                }
                run[tt] += node < cnt ? y : 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            cnt_r[j] = cnt_r[j + 1];
            dev_r[j] = dev_r[j + 1];
        }
    };
    for (int t = t_lo; t < t_hi; t += 2) {
        step(t, xb);
        if (t + 1 < t_hi) step(t + 1, xa);
    }
    flush();
    // device groups without a tile in this slice
    for (int d = 0; d < G; ++d) {
        if ((written >> d) & 1u) continue;
        for (int i = tid; i < H; i += kThreads) dst[d * H + i] = 0.0f;
    }
}

// ---- k_pool_stream: the same sums with every wave working on tiles of its own.
// One workgroup of eight waves per (set, graph); wave w is slice w of the set's tiles.  The
// weights of l_set sit in LDS as MFMA *A* operands (the products are taken transposed:
// out^T = W^T x^T), the sixteen nodes of a tile are the columns of the B operand:
//   * lane (n = lane % 16, g = lane / 16) loads eight floats of node n's row per k-step straight
//     from HBM (two 16-byte loads, issued kLoadAhead k-steps before their use), splits them exactly
//     into three bf16 parts in registers and uses them as B operands: the input never passes
//     through LDS, and there is no barrier in the tile loop;
//   * a weight fragment read from LDS serves the three parts; their products accumulate in one
//     accumulator, so the parts are summed by the matrix core;
//   * the transposed result of layer 1 (lane (n, g) holds columns 16 mt + 4 g + j of node n) is, with
//     two column tiles taken together, exactly a B operand of layer 2 for a permuted contraction
//     index (the packed weights of layer 2 carry the permutation): the activations go from one
//     layer to the next in registers;
//   * a lane adds its node's outputs to running sums; the sixteen lanes of a column are added in a
//     fixed order when the device group changes.
constexpr int kStreamWaves = 8;
constexpr int kStreamGraphsPerChip = 256;  // compute units of the chip: a workgroup of the streaming kernel fills one
constexpr int kStreamThreads = 64 * kStreamWaves;

// position in a row of the i-th of the eight values that lane group g holds in k-step ks
__host__ __device__ constexpr int stream_k(int ks, int g, int i) { return 32 * ks + 16 * (i / 4) + 4 * g + i % 4; }

template <int H, int L, bool KEEP = false>
__global__ __launch_bounds__(kStreamThreads, 1) void k_pool_stream(PoolParams P)
{
    constexpr int K1 = 2 * H;
    constexpr int KS1 = K1 / 32, KS2 = H / 32, MT = H / 16;
#ifndef PL_POOL_AHEAD
#define PL_POOL_AHEAD 4
#endif
    constexpr int kLoadAhead = KS1 < PL_POOL_AHEAD ? KS1 : PL_POOL_AHEAD;     // k-steps of input rows in flight
    constexpr int MG = MT < 4 ? MT : 4;               // column tiles whose chains interleave
#ifndef PL_POOL_INTERLEAVE
#define PL_POOL_INTERLEAVE 1
#endif
    constexpr bool kInterleave = PL_POOL_INTERLEAVE;
    constexpr int kFrags = MT * KS1 + (L > 1 ? MT * KS2 : 0);
    static_assert(KS1 % kLoadAhead == 0 && MT % MG == 0 && MT % 2 == 0, "shape");

    __shared__ uint4 wlds[kFrags * 64];               // A fragments of l_set: layer 1 [mt][ks], then layer 2
    __shared__ __attribute__((aligned(16))) float blds[L * H];
    __shared__ int kofs[kMaxD + 1];                   // first position of each device group of this set

    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // uniform: the tile walk stays in scalar registers
    const int n = lane & 15, g = lane >> 4;
    const GraphView &gv = P.gv;
    const int g0 = gv.node_off[b], g_n = gv.node_off[b + 1] - g0;
    const int G = P.G;
    int slices = (g_n + kPoolChunk - 1) / kPoolChunk;
    if (slices > P.max_slices) slices = P.max_slices;
    // A workgroup takes the sets blockIdx.x, blockIdx.x + gridDim.x, ..: all three of its graph
    // (grid.x = 1: every workgroup then has the same share of a batch of equal graphs, whatever
    // the sizes of the sets) or one (grid.x = 3, for batches that would not fill the chip otherwise).
    for (int set = blockIdx.x; set < 3; set += gridDim.x) {
    if (set != static_cast<int>(blockIdx.x)) __syncthreads();   // every wave is done with the weights of the previous set
    const int32_t *kb = P.koff + static_cast<size_t>(b) * (kMaxKeys + 1) + set * G;
    int n_tiles = 0;
    for (int d = 0; d < G; ++d) n_tiles += (kb[d + 1] - kb[d] + kBatch - 1) / kBatch;
    if (tid <= G) kofs[tid] = kb[tid];

    // The set's weights travel to LDS through registers, all loads in flight together; a wave's
    // first node ids and rows are requested before it waits for them.
    constexpr int kWPer = kFrags * 64 / kStreamThreads;
    static_assert(kFrags * 64 % kStreamThreads == 0, "fragments must divide over the threads");
    uint4 wtmp[kWPer];
    {
        const uint4 *src = P.wfrag + static_cast<size_t>(set) * kFrags * 64;
#pragma unroll
        for (int k = 0; k < kWPer; ++k) wtmp[k] = src[tid + k * kStreamThreads];
    }
    const bool idle = wave >= slices;
    const int t_lo = idle ? 0 : static_cast<int>(static_cast<long long>(n_tiles) * wave / slices);
    const int t_hi = idle ? 0 : static_cast<int>(static_cast<long long>(n_tiles) * (wave + 1) / slices);
    float *dst = P.partial + (((static_cast<size_t>(b) * P.max_slices + wave) * 3 + set) * G) * H;

    // ---- tile walk (uniform over the wave, offsets from LDS so that it never waits for loads from
    // HBM): device group w_dev, position w_pos of the walk's tile, w_left nodes of the group from there
    // (before the workgroup's barrier the offsets come from HBM, kof_g; afterwards from LDS, kof)
    auto kof = [&](int d) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(kofs[d]); };
    auto kof_g = [&](int d) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(kb[d]); };
    int w_dev = 0, w_pos = 0, w_left = 0;
    if (t_lo < t_hi) {                            // the device group of the slice's first tile
        int before = 0;
        for (;; ++w_dev) {
            const int tiles = (kof_g(w_dev + 1) - kof_g(w_dev) + kBatch - 1) / kBatch;
            if (t_lo < before + tiles) break;
            before += tiles;
        }
        w_pos = kof_g(w_dev) + (t_lo - before) * kBatch;
        w_left = kof_g(w_dev + 1) - w_pos;
    }
    // node of this lane in the walk's tile (rows past the tile's end repeat its first node); the
    // walk moves on to the next tile
    auto tile_next = [&](auto offsets, int &cnt, int &dev) __attribute__((always_inline)) {
        cnt = min(kBatch, w_left);
        dev = w_dev;
        const int id = P.klist[g0 + w_pos + (n < cnt ? n : 0)];
        w_pos += kBatch;
        w_left -= kBatch;
        while (w_left <= 0 && w_dev + 1 < G) {
            ++w_dev;
            w_pos = offsets(w_dev);
            w_left = offsets(w_dev + 1) - w_pos;
        }
        return id;
    };
    auto load_step = [&](int node, int ks, f32x4 (&x)[2]) __attribute__((always_inline)) {
        const float *row = P.emb + static_cast<size_t>(node) * K1 + 32 * ks + 4 * g;
        x[0] = *reinterpret_cast<const f32x4 *>(row);
        x[1] = *reinterpret_cast<const f32x4 *>(row + 16);
    };
    // exact three-way split of eight floats into bf16 parts (truncation), as MFMA operands
    auto split8 = [&](const float (&x)[8], bf16x8 (&part)[3]) __attribute__((always_inline)) {
        uint32_t w[3][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a0 = x[2 * q], a1 = x[2 * q + 1];
            const float r0 = a0 - trunc_bf16(a0), r1 = a1 - trunc_bf16(a1);
            const float l0 = r0 - trunc_bf16(r0), l1 = r1 - trunc_bf16(r1);
            w[0][q] = pack_hi16(a0, a1);
            w[1][q] = pack_hi16(r0, r1);
            w[2][q] = pack_hi16(l0, l1);
        }
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const uint4 v{w[p][0], w[p][1], w[p][2], w[p][3]};
            part[p] = *reinterpret_cast<const bf16x8 *>(&v);
        }
    };
    auto frag1 = [&](int mt, int ks) __attribute__((always_inline)) {
        const uint4 v = wlds[(mt * KS1 + ks) * 64 + lane];
        return *reinterpret_cast<const bf16x8 *>(&v);
    };
    auto frag2 = [&](int mt, int ks) __attribute__((always_inline)) {
        const uint4 v = wlds[(MT * KS1 + mt * KS2 + ks) * 64 + lane];
        return *reinterpret_cast<const bf16x8 *>(&v);
    };
    // The matrix instructions run in groups of MG column tiles x (hi, mid, lo) with one weight
    // fragment per tile, so that none waits for the one before it on the same accumulator.  Groups
    // are numbered through both layers: q < NG1: layer 1, k-step q / GPK, tiles MG (q % GPK) ..;
    // then layer 2 likewise.  The fragments of group q + 1 are read from LDS before the matrix
    // instructions of group q are issued.
    constexpr int GPK = MT / MG;                       // groups per k-step
    constexpr int NG1 = KS1 * GPK, NG = NG1 + (L > 1 ? KS2 * GPK : 0);
    auto read_group = [&](int q, bf16x8 (&a)[MG]) __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < MG; ++m)
            a[m] = q < NG1 ? frag1(MG * (q % GPK) + m, q / GPK) : frag2(MG * ((q - NG1) % GPK) + m, (q - NG1) / GPK);
    };
    auto mfma_group = [&](int m0, const bf16x8 (&a)[MG], const bf16x8 (&part)[3], f32x4 (&acc)[MT]) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < 3; ++p)
#pragma unroll
            for (int m = 0; m < MG; ++m)
                acc[m0 + m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[m], part[p], acc[m0 + m], 0, 0, 0);
    };

    f32x4 sum[MT];            // running sums of this lane's node slot over the tiles of the current device group
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) sum[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
    unsigned written = 0;
    // Adds the sixteen lanes of a column in a fixed order and writes the device group's sums.
    auto row_sum = [](float v) __attribute__((always_inline)) {
        auto step = [](float x, auto ctrl) __attribute__((always_inline)) {
            return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, false));
        };
        v = step(v, std::integral_constant<int, 0xB1>{});     // quad_perm [1, 0, 3, 2]
        v = step(v, std::integral_constant<int, 0x4E>{});     // quad_perm [2, 3, 0, 1]
        v = step(v, std::integral_constant<int, 0x141>{});    // row_half_mirror
        v = step(v, std::integral_constant<int, 0x140>{});    // row_mirror
        return v;
    };
    auto flush = [&](int dev_done) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            f32x4 sv;
#pragma unroll
            for (int j = 0; j < 4; ++j) sv[j] = row_sum(sum[mt][j]);
            if (n == 0) *reinterpret_cast<f32x4 *>(dst + dev_done * H + 16 * mt + 4 * g) = sv;
            sum[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
        written |= 1u << dev_done;
    };

    // ---- pipeline: the rows of k-step s + kLoadAhead are in flight while k-step s is computed
    // The node ids of tile t + 2 are fetched at the start of tile t, before that tile's row loads:
    // loads return in order, so when an id is handed on at the end of a tile it arrived long ago
    // and the wait for it leaves the row loads in flight.
    f32x4 raw[kLoadAhead][2];
    int cnt = 0, dev = 0, cnt_next = 0, dev_next = 0, cnt_after = 0, dev_after = 0;
    int node = g0, node_next = g0, node_after = g0;
    if (t_lo < t_hi) {
        node = node_next = node_after = tile_next(kof_g, cnt, dev);
        if (t_lo + 1 < t_hi) node_next = tile_next(kof_g, cnt_next, dev_next);
#pragma unroll
        for (int ks = 0; ks < kLoadAhead; ++ks) load_step(node, ks, raw[ks]);
    }
    // ---- the weights arrive: every wave writes its share, then the workgroup meets
#pragma unroll
    for (int k = 0; k < kWPer; ++k) wlds[tid + k * kStreamThreads] = wtmp[k];
    for (int i = tid; i < L * H; i += kStreamThreads) blds[i] = P.bias[set * L * H + i];
    __syncthreads();
    if (idle) continue;
    if (t_lo >= t_hi) {
        for (int i = lane; i < G * H; i += 64) dst[i] = 0.0f;
        continue;
    }
    bf16x8 afr[2][MG];
    read_group(0, afr[0]);
    // nothing loaded before the loop is in flight when it starts, so that the waits inside the
    // loop are counted from the loop's own loads alone
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)

    int t = t_lo;
    while (t < t_hi) {
        const int seg_dev = dev;
        // the tiles of one device group
        for (;;) {
            const bool more = t + 1 < t_hi;
            if (t + 2 < t_hi) node_after = tile_next(kof, cnt_after, dev_after);
            f32x4 acc[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) acc[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
            // ---- layer 1.  The split of k-step ks + 1 and the loads of k-step ks + kLoadAhead are
            // written before the matrix instructions of k-step ks and interleaved with them by the
            // scheduling groups below: the vector unit works while the matrix core is busy.
            bf16x8 part[2][3];
            {
                float x[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) x[i] = raw[0][i / 4][i % 4];
                split8(x, part[0]);
            }
#pragma unroll
            for (int ks = 0; ks < KS1; ++ks) {
                // (after the slice's last tile the same rows once more: every path issues the
                // same loads, so the waits for them are counted exactly)
                if (ks + kLoadAhead < KS1)
                    load_step(node, ks + kLoadAhead, raw[ks % kLoadAhead]);
                else
                    load_step(more ? node_next : node, ks + kLoadAhead - KS1, raw[ks % kLoadAhead]);
                if (ks + 1 < KS1) {
                    float x[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) x[i] = raw[(ks + 1) % kLoadAhead][i / 4][i % 4];
                    split8(x, part[(ks + 1) & 1]);
                }
#pragma unroll
                for (int gq = 0; gq < GPK; ++gq) {
                    const int q = ks * GPK + gq;
                    read_group((q + 1) % NG, afr[(q + 1) & 1]);
                    mfma_group(MG * gq, afr[q & 1], part[ks & 1], acc);
                }
                if constexpr (kInterleave) {
                    __builtin_amdgcn_sched_group_barrier(0x020, 2, 0);      // the two row loads
#pragma unroll
                    for (int gq = 0; gq < GPK; ++gq) {
                        __builtin_amdgcn_sched_group_barrier(0x100, MG, 0); // fragments of the next group
#pragma unroll
                        for (int i = 0; i < 3 * MG; ++i) {
                            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                            __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                        }
                    }
                }
            }
            // ---- bias, ReLU; layer 2 from registers
            f32x4 out[MT];
            if constexpr (L > 1) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) out[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
                // bias, ReLU and split of the two column tiles that k-step ks of layer 2 contracts
                auto hand_on = [&](int ks, bf16x8 (&pt)[3]) __attribute__((always_inline)) {
                    float y[8];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int mt = 2 * ks + h;
                        const f32x4 bv = *reinterpret_cast<const f32x4 *>(&blds[16 * mt + 4 * g]);
                        f32x4 yy;
#pragma unroll
                        for (int j = 0; j < 4; ++j) yy[j] = y[4 * h + j] = fmaxf(acc[mt][j] + bv[j], 0.0f);
                        if constexpr (KEEP) {
                            if (n < cnt) *reinterpret_cast<f32x4 *>(P.keep + static_cast<size_t>(node) * H + 16 * mt + 4 * g) = yy;
                        }
                    }
                    split8(y, pt);
                };
                hand_on(0, part[0]);
#pragma unroll
                for (int ks = 0; ks < KS2; ++ks) {
                    if (ks + 1 < KS2) hand_on(ks + 1, part[(ks + 1) & 1]);
#pragma unroll
                    for (int gq = 0; gq < GPK; ++gq) {
                        const int q = NG1 + ks * GPK + gq;
                        read_group((q + 1) % NG, afr[(q + 1) & 1]);
                        mfma_group(MG * gq, afr[q & 1], part[ks & 1], out);
                    }
                    if constexpr (kInterleave && !KEEP) {
#pragma unroll
                        for (int gq = 0; gq < GPK; ++gq) {
                            if (gq == 0) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // the biases
                            __builtin_amdgcn_sched_group_barrier(0x100, MG, 0);
#pragma unroll
                            for (int i = 0; i < 3 * MG; ++i) {
                                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                                __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
                            }
                        }
                    }
                }
            } else {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) out[mt] = acc[mt];
            }
            // ---- bias, ReLU of the last layer; the node's outputs join the running sums
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                const f32x4 bv = *reinterpret_cast<const f32x4 *>(&blds[(L - 1) * H + 16 * mt + 4 * g]);
                f32x4 yy;
#pragma unroll
                for (int j = 0; j < 4; ++j) yy[j] = fmaxf(out[mt][j] + bv[j], 0.0f);
                if constexpr (KEEP) {
                    if (n < cnt)
                        *reinterpret_cast<f32x4 *>(P.keep + (static_cast<size_t>(L - 1) * gv.n_tot + node) * H + 16 * mt + 4 * g) = yy;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) sum[mt][j] += n < cnt ? yy[j] : 0.0f;
            }
            node = node_next;
            cnt = cnt_next;
            dev = dev_next;
            node_next = node_after;
            cnt_next = cnt_after;
            dev_next = dev_after;
            ++t;
            if (t >= t_hi || dev != seg_dev) break;
        }
        flush(seg_dev);
    }
    for (int d = 0; d < G; ++d) {
        if ((written >> d) & 1u) continue;
        for (int i = lane; i < H; i += 64) dst[d * H + i] = 0.0f;
    }
    }   // sets
}

// ---- k_pool_stream_bw: the reverse of k_pool_stream for two-layer l networks, one pass over the
// tiles that the forward pass pooled (same sort, same slices):
//   delta2 = dP[set][device] gated by l's output, delta1 = (W2 delta2) gated by the first layer's
//   output, d e = W1 delta1,
// with the products taken transposed as in the forward kernel: the weights (as stored: row i of a
// layer holds the outputs fed by input i) are the A operands in LDS, a tile's sixteen nodes the
// columns of the B operand, deltas split exactly into three bf16 parts, the result of the first
// product chained into the second in registers.  Both deltas are also written out for the weight
// gradients.  Nodes that were pooled nowhere (device id out of range) are not visited:
// k_zero_unpooled clears their rows.
struct PoolBwParams {
    GraphView gv;
    const uint4 *wfrag;        // see pack_pool_stream_bw_weights
    const float *keep;         // [2][n_tot, H] outputs of l's layers (written by the forward pooling kernel)
    const float *dP;           // [B, 3, G, H] gradient of the pooled sums
    const int32_t *klist;
    const int32_t *koff;
    float *dl;                 // [2][n_tot, H] deltas of l's layers
    float *demb;               // [n_tot, 2H]
    int max_slices;
    int G;
};

template <int H>
__global__ __launch_bounds__(kStreamThreads, 1) void k_pool_stream_bw(PoolBwParams P)
{
    constexpr int K1 = 2 * H;
    constexpr int KS = H / 32, MT2 = H / 16, MT1 = K1 / 16;   // both products contract over H
    constexpr int MG = 4;
    constexpr int kFrags = MT2 * KS + MT1 * KS;
    static_assert(MT2 % MG == 0 && MT1 % MG == 0 && KS == 4, "shape");

    __shared__ uint4 wlds[kFrags * 64];               // A fragments: W2 [mt][ks], then W1 [mt][ks]
    __shared__ __attribute__((aligned(16))) float dplds[kMaxD * H];   // dP of this (graph, set)
    __shared__ int kofs[kMaxD + 1];

    const int b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 15, g = lane >> 4;
    const GraphView &gv = P.gv;
    const int g0 = gv.node_off[b], g_n = gv.node_off[b + 1] - g0;
    const int G = P.G;
    const size_t NH = static_cast<size_t>(gv.n_tot) * H;
    int slices = (g_n + kPoolChunk - 1) / kPoolChunk;
    if (slices > P.max_slices) slices = P.max_slices;
    for (int set = blockIdx.x; set < 3; set += gridDim.x) {
    if (set != static_cast<int>(blockIdx.x)) __syncthreads();
    const int32_t *kb = P.koff + static_cast<size_t>(b) * (kMaxKeys + 1) + set * G;
    int n_tiles = 0;
    for (int d = 0; d < G; ++d) n_tiles += (kb[d + 1] - kb[d] + kBatch - 1) / kBatch;
    if (tid <= G) kofs[tid] = kb[tid];
    constexpr int kWPer = kFrags * 64 / kStreamThreads;
    static_assert(kFrags * 64 % kStreamThreads == 0, "fragments must divide over the threads");
    {
        uint4 wtmp[kWPer];
        const uint4 *src = P.wfrag + static_cast<size_t>(set) * kFrags * 64;
#pragma unroll
        for (int k = 0; k < kWPer; ++k) wtmp[k] = src[tid + k * kStreamThreads];
#pragma unroll
        for (int k = 0; k < kWPer; ++k) wlds[tid + k * kStreamThreads] = wtmp[k];
    }
    for (int i = tid; i < G * H; i += kStreamThreads)
        dplds[i] = P.dP[((static_cast<size_t>(b) * 3 + set) * G) * H + i];
    __syncthreads();
    if (wave >= slices) continue;
    const int t_lo = static_cast<int>(static_cast<long long>(n_tiles) * wave / slices);
    const int t_hi = static_cast<int>(static_cast<long long>(n_tiles) * (wave + 1) / slices);
    if (t_lo >= t_hi) continue;

    auto kof = [&](int d) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(kofs[d]); };
    int w_dev = 0, w_pos = 0, w_left = 0;
    {
        int before = 0;
        for (;; ++w_dev) {
            const int tiles = (kof(w_dev + 1) - kof(w_dev) + kBatch - 1) / kBatch;
            if (t_lo < before + tiles) break;
            before += tiles;
        }
        w_pos = kof(w_dev) + (t_lo - before) * kBatch;
        w_left = kof(w_dev + 1) - w_pos;
    }
    auto tile_next = [&](int &cnt, int &dev) __attribute__((always_inline)) {
        cnt = min(kBatch, w_left);
        dev = w_dev;
        const int id = P.klist[g0 + w_pos + (n < cnt ? n : 0)];
        w_pos += kBatch;
        w_left -= kBatch;
        while (w_left <= 0 && w_dev + 1 < G) {
            ++w_dev;
            w_pos = kof(w_dev);
            w_left = kof(w_dev + 1) - w_pos;
        }
        return id;
    };
    auto split8 = [&](const float (&x)[8], bf16x8 (&part)[3]) __attribute__((always_inline)) {
        uint32_t w[3][4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float a0 = x[2 * q], a1 = x[2 * q + 1];
            const float r0 = a0 - trunc_bf16(a0), r1 = a1 - trunc_bf16(a1);
            const float l0 = r0 - trunc_bf16(r0), l1 = r1 - trunc_bf16(r1);
            w[0][q] = pack_hi16(a0, a1);
            w[1][q] = pack_hi16(r0, r1);
            w[2][q] = pack_hi16(l0, l1);
        }
#pragma unroll
        for (int p = 0; p < 3; ++p) {
            const uint4 v{w[p][0], w[p][1], w[p][2], w[p][3]};
            part[p] = *reinterpret_cast<const bf16x8 *>(&v);
        }
    };
    // groups of MG row tiles of the result, numbered through both products: q < NG2: W2, k-step
    // q / GP2; then W1, k-step (q - NG2) / GP1
    constexpr int GP2 = MT2 / MG, GP1 = MT1 / MG, NG2 = KS * GP2, NG = NG2 + KS * GP1;
    auto read_group = [&](int q, bf16x8 (&a)[MG]) __attribute__((always_inline)) {
#pragma unroll
        for (int m = 0; m < MG; ++m) {
            const int f = q < NG2 ? (MG * (q % GP2) + m) * KS + q / GP2
                                  : MT2 * KS + (MG * ((q - NG2) % GP1) + m) * KS + (q - NG2) / GP1;
            const uint4 v = wlds[f * 64 + lane];
            a[m] = *reinterpret_cast<const bf16x8 *>(&v);
        }
    };
    // the eight gate values (layer outputs) of this lane for k-step ks of a row of `base`
    auto load_step = [&](const float *base, int node, int ks, f32x4 (&x)[2]) __attribute__((always_inline)) {
        const float *row = base + static_cast<size_t>(node) * H + 32 * ks + 4 * g;
        x[0] = *reinterpret_cast<const f32x4 *>(row);
        x[1] = *reinterpret_cast<const f32x4 *>(row + 16);
    };

    const float *keep1 = P.keep, *keep2 = P.keep + NH;
    float *dl1 = P.dl, *dl2 = P.dl + NH;
    f32x4 y2[KS][2];           // l's outputs of the tile in flight (gates of delta2), one tile ahead
    int cnt = 0, dev = 0, cnt_next = 0, dev_next = 0, cnt_after = 0, dev_after = 0;
    int node = tile_next(cnt, dev);
    int node_next = node, node_after = node;
    if (t_lo + 1 < t_hi) node_next = tile_next(cnt_next, dev_next);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) load_step(keep2, node, ks, y2[ks]);
    bf16x8 afr[2][MG];
    read_group(0, afr[0]);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the loop's waits are counted from its own loads

    for (int t = t_lo; t < t_hi; ++t) {
        const bool more = t + 1 < t_hi;
        const bool live = n < cnt;
        if (t + 2 < t_hi) node_after = tile_next(cnt_after, dev_after);
        // the first layer's outputs of this tile (gates of delta1): needed after the first product
        f32x4 y1[MT2];
#pragma unroll
        for (int mt = 0; mt < MT2; ++mt)
            y1[mt] = *reinterpret_cast<const f32x4 *>(keep1 + static_cast<size_t>(node) * H + 16 * mt + 4 * g);
        // ---- delta2 and the product with W2
        f32x4 acc1[MT2];
#pragma unroll
        for (int mt = 0; mt < MT2; ++mt) acc1[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            float d2[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const f32x4 dp = *reinterpret_cast<const f32x4 *>(&dplds[dev * H + 32 * ks + 16 * h + 4 * g]);
                f32x4 dv;
#pragma unroll
                for (int j = 0; j < 4; ++j) dv[j] = d2[4 * h + j] = y2[ks][h][j] > 0.0f ? dp[j] : 0.0f;
                if (live) *reinterpret_cast<f32x4 *>(dl2 + static_cast<size_t>(node) * H + 32 * ks + 16 * h + 4 * g) = dv;
            }
            // the same rows once more after the slice's last tile: every path issues the same loads
            load_step(keep2, more ? node_next : node, ks, y2[ks]);
            bf16x8 part[3];
            split8(d2, part);
#pragma unroll
            for (int gq = 0; gq < GP2; ++gq) {
                const int q = ks * GP2 + gq;
                read_group(q + 1, afr[(q + 1) & 1]);
                __builtin_amdgcn_sched_barrier(6);
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int m = 0; m < MG; ++m)
                        acc1[MG * gq + m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[q & 1][m], part[p], acc1[MG * gq + m], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(6);
            }
        }
        // ---- delta1 (gated), and the product with W1
        f32x4 acc0[MT1];
#pragma unroll
        for (int mt = 0; mt < MT1; ++mt) acc0[mt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            float d1[8];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int mt = 2 * ks + h;
                f32x4 dv;
#pragma unroll
                for (int j = 0; j < 4; ++j) dv[j] = d1[4 * h + j] = y1[mt][j] > 0.0f ? acc1[mt][j] : 0.0f;
                if (live) *reinterpret_cast<f32x4 *>(dl1 + static_cast<size_t>(node) * H + 16 * mt + 4 * g) = dv;
            }
            bf16x8 part[3];
            split8(d1, part);
#pragma unroll
            for (int gq = 0; gq < GP1; ++gq) {
                const int q = NG2 + ks * GP1 + gq;
                read_group((q + 1) % NG, afr[(q + 1) & 1]);
                __builtin_amdgcn_sched_barrier(6);
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int m = 0; m < MG; ++m)
                        acc0[MG * gq + m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afr[q & 1][m], part[p], acc0[MG * gq + m], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(6);
            }
        }
        if (live) {
#pragma unroll
            for (int mt = 0; mt < MT1; ++mt)
                *reinterpret_cast<f32x4 *>(P.demb + static_cast<size_t>(node) * K1 + 16 * mt + 4 * g) = acc0[mt];
        }
        node = node_next;
        cnt = cnt_next;
        dev = dev_next;
        node_next = node_after;
        cnt_next = cnt_after;
        dev_next = dev_after;
    }
    }   // sets
}

// Rows of the deltas of l and of d e for nodes that belong to a set but were pooled nowhere (device
// id out of range): zero.
__global__ __launch_bounds__(kThreads) void k_zero_unpooled(int n_tot, int H, int L, int D, const uint8_t *__restrict__ cls,
                                                            const int32_t *__restrict__ placement,
                                                            float *__restrict__ dl, float *__restrict__ demb)
{
    const int v = blockIdx.x * kThreads + threadIdx.x;
    if (v >= n_tot || cls[v] == 0) return;
    const int dev = placement[v];
    if (dev >= 0 && dev < D) return;
    for (int l = 0; l < L; ++l)
        for (int i = 0; i < H; ++i) dl[(static_cast<size_t>(l) * n_tot + v) * H + i] = 0.0f;
    for (int i = 0; i < 2 * H; ++i) demb[static_cast<size_t>(v) * 2 * H + i] = 0.0f;
}

// Appends the MFMA B-operand fragments of one layer: index ((nt * KS + ks) * WS + ws) * 64 + lane,
// lane l holds W[32 ks + 8 (l / 16) + i][16 nt + l % 16], i = 0..7, as bf16 part ws of the exact
// three-way split of the weight (ws = 0 only when the weights are bf16 already).
// With `paired` the contraction index follows the order in which a lane that owns two output
// columns of the previous layer writes them (columns c and c + 16 of a wave as the halves of one
// word): k = 32 ks + 16 (i % 2) + 4 (l / 16) + i / 2.
void append_fragments(const float *blob, const LayerRef &lr, int WS, std::vector<uint16_t> *out, bool paired = false)
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
                    const int k = paired ? 32 * ks + 16 * (i % 2) + 4 * (lane / 16) + i / 2 : 32 * ks + 8 * (lane / 16) + i;
                    const int m = 16 * nt + lane % 16;
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
            append_fragments(blob, mv.l[set].layer[l], WS, frag, l > 0 && (mv.H / 16 + 3) / 4 == 2);
            for (int h = 0; h < mv.H; ++h)
                (*bias)[(static_cast<size_t>(set) * mv.L + l) * mv.H + h] = blob[mv.l[set].layer[l].b + h];
        }
}

// A fragments of the streaming kernel: per set, layer 1 [mt][ks] then layer 2 [mt][ks], 64 lanes
// of eight bf16: lane l holds W[stream_k(ks, l / 16, i)][16 mt + l % 16], i = 0..7 (bf16 weights).
void pack_pool_stream_weights(const ModelView &mv, const float *blob, std::vector<uint16_t> *frag)
{
    frag->clear();
    auto to_bf16 = [](float x) {
        uint32_t u;
        std::memcpy(&u, &x, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return static_cast<uint16_t>(u >> 16);
    };
    for (int set = 0; set < 3; ++set)
        for (int l = 0; l < mv.L; ++l) {
            const LayerRef &lr = mv.l[set].layer[l];
            const int MT = lr.n_out / 16, KS = lr.n_in / 32;
            for (int mt = 0; mt < MT; ++mt)
                for (int ks = 0; ks < KS; ++ks)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int i = 0; i < 8; ++i) {
                            const int k = stream_k(ks, lane / 16, i), m = 16 * mt + lane % 16;
                            frag->push_back(to_bf16(blob[lr.w + static_cast<size_t>(k) * lr.n_out + m]));
                        }
        }
}

// A fragments of the reverse streaming kernel (two-layer l): per set, W2 [mt][ks] then W1 [mt][ks];
// lane l holds W[16 mt + l % 16][stream_k(ks, l / 16, i)], i = 0..7: row = the layer's input index,
// the contraction runs over its outputs.
void pack_pool_stream_bw_weights(const ModelView &mv, const float *blob, std::vector<uint16_t> *frag)
{
    frag->clear();
    auto to_bf16 = [](float x) {
        uint32_t u;
        std::memcpy(&u, &x, 4);
        u += 0x7FFFu + ((u >> 16) & 1u);
        return static_cast<uint16_t>(u >> 16);
    };
    for (int set = 0; set < 3; ++set)
        for (int l = mv.L - 1; l >= 0; --l) {
            const LayerRef &lr = mv.l[set].layer[l];
            const int MT = lr.n_in / 16, KS = lr.n_out / 32;
            for (int mt = 0; mt < MT; ++mt)
                for (int ks = 0; ks < KS; ++ks)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int i = 0; i < 8; ++i) {
                            const int k = stream_k(ks, lane / 16, i), m = 16 * mt + lane % 16;
                            frag->push_back(to_bf16(blob[lr.w + static_cast<size_t>(m) * lr.n_out + k]));
                        }
        }
}

bool pool_stream_bw_supported(int H, int L, int weight_dtype)
{
    return weight_dtype == PL_WEIGHTS_BF16 && H == 128 && L == 2;
}

void launch_pool_stream_bw(const GraphView &gv, const ModelView &mv, const Workspace &ws, const int32_t *placement,
                           const uint4 *frag, const float *lact, const float *dP, const uint8_t *cls, float *dl,
                           float *demb, hipStream_t s)
{
    if (gv.B == 0) return;
    hipLaunchKernelGGL(k_zero_unpooled, dim3((gv.n_tot + kThreads - 1) / kThreads), dim3(kThreads), 0, s, gv.n_tot, mv.H,
                       mv.L, mv.D, cls, placement, dl, demb);
    PoolBwParams P{gv, frag, lact, dP, ws.klist, ws.koff, dl, demb, kStreamWaves, mv.G};
    const dim3 grid(gv.B < kStreamGraphsPerChip ? 3 : 1, gv.B), block(kStreamThreads);
    hipLaunchKernelGGL((k_pool_stream_bw<128>), grid, block, 0, s, P);
}

bool pool_stream_supported(int H, int L, int weight_dtype)
{
    return weight_dtype == PL_WEIGHTS_BF16 && H == 128 && (L == 1 || L == 2);
}

bool pool_mfma_supported(int H, int L, int weight_dtype)
{
    if (L < 1 || L > 2) return false;
    if (weight_dtype == PL_WEIGHTS_BF16) return H == 32 || H == 64 || H == 128;
    return H == 32 || H == 64;
}

int launch_pool_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                     const ForwardArgs &fa, const uint4 *wfrag, const uint4 *afrag, const float *bias, int WS,
                     float *keep, hipStream_t s)
{
    if (gv.B == 0) return kPoolSlices;
    hipLaunchKernelGGL(k_pool_sort, dim3(gv.B), dim3(kThreads), 0, s, gv, ws.reach, fa.placement, fa.cur_node, mv.D,
                       mv.G, mv.single_set, ws.klist, ws.koff);
    // the shapes that the streaming kernel covers take it (eight slices per set, one per wave)
    if (afrag && WS == 1 && pool_stream_supported(mv.H, mv.L, PL_WEIGHTS_BF16)) {
        PoolParams Q{gv, afrag, bias, ws.emb, ws.klist, ws.koff, ws.partial, kStreamWaves, mv.G, keep};
        // one workgroup per graph once that fills the chip; a workgroup per (set, graph) below
        const dim3 grid(gv.B < kStreamGraphsPerChip ? 3 : 1, gv.B), block(kStreamThreads);
        if (mv.L == 2) {
            if (keep)
                hipLaunchKernelGGL((k_pool_stream<128, 2, true>), grid, block, 0, s, Q);
            else
                hipLaunchKernelGGL((k_pool_stream<128, 2>), grid, block, 0, s, Q);
        } else {
            if (keep)
                hipLaunchKernelGGL((k_pool_stream<128, 1, true>), grid, block, 0, s, Q);
            else
                hipLaunchKernelGGL((k_pool_stream<128, 1>), grid, block, 0, s, Q);
        }
        return kStreamWaves;
    }
    PoolParams P{gv, wfrag, bias, ws.emb, ws.klist, ws.koff, ws.partial, kPoolSlices, mv.G, keep};
    const dim3 grid(3, kPoolSlices, gv.B), block(kThreads);
#define PL_CASE(HH, WW, LL)                                                          \
    if (mv.H == HH && WS == WW && mv.L == LL) {                                      \
        if (keep)                                                                    \
            hipLaunchKernelGGL((k_pool_tiles<HH, WW, LL, true>), grid, block, 0, s, P); \
        else                                                                         \
            hipLaunchKernelGGL((k_pool_tiles<HH, WW, LL>), grid, block, 0, s, P);    \
        return kPoolSlices;                                                          \
    }
    PL_CASE(64, 1, 2) PL_CASE(64, 1, 1) PL_CASE(64, 3, 2) PL_CASE(64, 3, 1)
    PL_CASE(32, 1, 2) PL_CASE(32, 1, 1) PL_CASE(32, 3, 2) PL_CASE(32, 3, 1)
#undef PL_CASE
    return kPoolSlices;
}

}  // namespace pl
