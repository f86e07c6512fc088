// Generic fp32 kernels for the policy forward pass: any H <= 256, D <= 16, 1..4 layers.
// They are the reference-quality HIP path (plain vector FMAs, deterministic summation
// order) and the fallback for shapes the matrix-core kernels do not cover.
//
// Section 2.2 of the paper: (1) raw features, (2) two-way message passing
// x_v <- g(sum_{u in xi(v)} f(x_u)), (3) pooling h_i(sum_{u in S_i(v)} l_i(x_u)) over the
// parent / child / parallel sets of the current node, then the policy head (Appendix A.7).
#include <type_traits>

#include "internal.h"

namespace pl {

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 16;   // rows (nodes) pushed through a network together

// y[r][j] = act(bias[j] + sum_k x[r][k] * W[k][j]) for r < rows (rows <= kTile).
// x and y live in LDS.  Thread (grp, j): column j = tid % n_out, row group grp = tid / n_out;
// it owns rows grp, grp + groups, ... (at most RPT of them), so one weight load feeds up to
// RPT FMAs.  Requires n_out <= kThreads and min(kThreads / n_out, kTile) * RPT >= rows.
template <int RPT, bool WIDE = false, int KL = 16>
__device__ __forceinline__ void dense_layer(const float *__restrict__ W,
                                            const float *__restrict__ bias, int n_in, int n_out,
                                            const float *x, int ldx, float *y, int ldy, int rows,
                                            bool relu)
{
    const int tid = threadIdx.x;
    int groups = kThreads / n_out;
    if (groups > kTile) groups = kTile;
    const int grp = tid / n_out, j = tid - grp * n_out;
    if (grp >= groups || grp >= rows) return;
    // WIDE: blocks of sixteen fp32 terms are added up in float64 (the policy head's networks,
    // whose inputs are sums over thousands of nodes)
    typedef typename std::conditional<WIDE, double, float>::type acc_t;
    acc_t acc[RPT];
    const float bj = bias[j];
#pragma unroll
    for (int i = 0; i < RPT; ++i) acc[i] = bj;
    int xoff[RPT];   // rows past the tile's end re-read its last row (never stored)
#pragma unroll
    for (int i = 0; i < RPT; ++i) xoff[i] = min(grp + i * groups, rows - 1) * ldx;
    // weights KL at a time, all loads issued before the first use: the loop is bound by the
    // latency of one batch instead of one load per step.  (WIDE: the float64 blocks stay sixteen
    // terms long whatever KL is.)
    constexpr int KB = 16;
    static_assert(KL % KB == 0, "a batch of loads is a whole number of blocks");
    int k = 0;
    for (; k + KL <= n_in; k += KL) {
        float w[KL];
#pragma unroll
        for (int u = 0; u < KL; ++u) w[u] = W[static_cast<size_t>(k + u) * n_out + j];
        if constexpr (WIDE) {
#pragma unroll
            for (int u0 = 0; u0 < KL; u0 += KB) {
                float part[RPT];
#pragma unroll
                for (int i = 0; i < RPT; ++i) part[i] = 0.0f;
#pragma unroll
                for (int u = u0; u < u0 + KB; ++u)
#pragma unroll
                    for (int i = 0; i < RPT; ++i) part[i] = fmaf(x[xoff[i] + k + u], w[u], part[i]);
#pragma unroll
                for (int i = 0; i < RPT; ++i) acc[i] += static_cast<double>(part[i]);
            }
            continue;
        }
#pragma unroll
        for (int u = 0; u < KL; ++u)
#pragma unroll
            for (int i = 0; i < RPT; ++i) acc[i] = fmaf(x[xoff[i] + k + u], w[u], acc[i]);
    }
    if constexpr (KL > KB) {          // whole blocks left over
        for (; k + KB <= n_in; k += KB) {
            float w[KB];
#pragma unroll
            for (int u = 0; u < KB; ++u) w[u] = W[static_cast<size_t>(k + u) * n_out + j];
            if constexpr (WIDE) {
                float part[RPT];
#pragma unroll
                for (int i = 0; i < RPT; ++i) part[i] = 0.0f;
#pragma unroll
                for (int u = 0; u < KB; ++u)
#pragma unroll
                    for (int i = 0; i < RPT; ++i) part[i] = fmaf(x[xoff[i] + k + u], w[u], part[i]);
#pragma unroll
                for (int i = 0; i < RPT; ++i) acc[i] += static_cast<double>(part[i]);
            } else {
#pragma unroll
                for (int u = 0; u < KB; ++u)
#pragma unroll
                    for (int i = 0; i < RPT; ++i) acc[i] = fmaf(x[xoff[i] + k + u], w[u], acc[i]);
            }
        }
    }
    for (; k < n_in; ++k) {
        const float w = W[static_cast<size_t>(k) * n_out + j];
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            if constexpr (WIDE)
                acc[i] += static_cast<double>(x[xoff[i] + k]) * static_cast<double>(w);
            else
                acc[i] = fmaf(x[xoff[i] + k], w, acc[i]);
        }
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = grp + i * groups;
        const float out = static_cast<float>(acc[i]);
        if (r < rows) y[r * ldy + j] = relu ? fmaxf(out, 0.0f) : out;
    }
}

// ------------------------------------------------------------------ step 1: features
// phi_v = [time, size, one-hot(device), is-current, is-visited]; x_v = relu(W^T phi_v + b).
// The two directions start from the same x: it goes to both halves of the embedding
// (node order) and/or to the per-direction bucket-ordered input of the matrix-core sweep.
__global__ __launch_bounds__(kThreads) void k_project(GraphView gv, ModelView mv,
                                                      const float *__restrict__ feats,
                                                      const int32_t *__restrict__ placement,
                                                      const int32_t *__restrict__ cur_node,
                                                      float *__restrict__ emb,
                                                      float *__restrict__ xb)
{
    const int H = mv.H, D = mv.D;
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= static_cast<size_t>(gv.n_tot) * H) return;
    const int v = static_cast<int>(idx / H), h = static_cast<int>(idx - static_cast<size_t>(v) * H);
    const int b = gv.node_graph[v];
    const float *W = mv.blob + mv.proj.w;
    float s = mv.blob[mv.proj.b + h];
    s = fmaf(feats[v * 3 + 0], W[0 * H + h], s);
    s = fmaf(feats[v * 3 + 1], W[1 * H + h], s);
    const int dev = placement[v];
    if (dev >= 0 && dev < D) s += W[(2 + dev) * H + h];
    if (v - gv.node_off[b] == cur_node[b]) s += W[(2 + D) * H + h];
    s = fmaf(feats[v * 3 + 2], W[(3 + D) * H + h], s);
    s = fmaxf(s, 0.0f);
    if (emb) {
        emb[static_cast<size_t>(v) * 2 * H + h] = s;
        emb[static_cast<size_t>(v) * 2 * H + H + h] = s;
    }
    if (xb) {
        xb[static_cast<size_t>(gv.pos[0][v]) * H + h] = s;
        xb[(static_cast<size_t>(gv.n_tot) + gv.pos[1][v]) * H + h] = s;
    }
}

// The same with four columns per thread, for H a multiple of four (vector loads and stores; the
// terms are added in the same order).
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4j;
__global__ __launch_bounds__(kThreads) void k_project4(GraphView gv, ModelView mv,
                                                       const float *__restrict__ feats,
                                                       const int32_t *__restrict__ placement,
                                                       const int32_t *__restrict__ cur_node,
                                                       float *__restrict__ emb,
                                                       float *__restrict__ xb)
{
    const int H = mv.H, D = mv.D, q = H / 4;
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= static_cast<size_t>(gv.n_tot) * q) return;
    const int v = static_cast<int>(idx / q), h = 4 * static_cast<int>(idx - static_cast<size_t>(v) * q);
    const int b = gv.node_graph[v];
    const float *W = mv.blob + mv.proj.w;
    auto row = [&](int r) { return *reinterpret_cast<const f32x4j *>(W + static_cast<size_t>(r) * H + h); };
    const float f_time = feats[v * 3 + 0], f_size = feats[v * 3 + 1], f_vis = feats[v * 3 + 2];
    const int dev = placement[v];
    const bool on_dev = dev >= 0 && dev < D;
    const bool is_cur = v - gv.node_off[b] == cur_node[b];
    const f32x4j bias = *reinterpret_cast<const f32x4j *>(mv.blob + mv.proj.b + h);
    const f32x4j w0 = row(0), w1 = row(1), wd = row(2 + (on_dev ? dev : 0)), wc = row(2 + D), wv = row(3 + D);
    f32x4j out;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float s = bias[k];
        s = fmaf(f_time, w0[k], s);
        s = fmaf(f_size, w1[k], s);
        if (on_dev) s += wd[k];
        if (is_cur) s += wc[k];
        s = fmaf(f_vis, wv[k], s);
        out[k] = fmaxf(s, 0.0f);
    }
    if (emb) {
        *reinterpret_cast<f32x4j *>(emb + static_cast<size_t>(v) * 2 * H + h) = out;
        *reinterpret_cast<f32x4j *>(emb + static_cast<size_t>(v) * 2 * H + H + h) = out;
    }
    if (xb) {
        *reinterpret_cast<f32x4j *>(xb + static_cast<size_t>(gv.pos[0][v]) * H + h) = out;
        *reinterpret_cast<f32x4j *>(xb + (static_cast<size_t>(gv.n_tot) + gv.pos[1][v]) * H + h) = out;
    }
}

// ------------------------------------------------------------------ step 2: one sweep
// One workgroup per (graph, direction) walks the graph's levels in order; graphs are
// independent, so no grid-wide barrier is needed.  For every node v of a level:
//   a_v = sum over neighbours u (parents top-down, children bottom-up) of m_u
//   s_v <- s_v + g(a_v);  m_v = f(s_v)
// and, riding along, the reachability bit used for the node sets of step 3:
//   top-down:  desc(v) = OR over parents p of (p == v* or desc(p))
//   bottom-up: anc(v)  = OR over children c of (c == v* or anc(c))
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_sweep_generic(GraphView gv, ModelView mv,
                                                            float *__restrict__ emb,
                                                            float *__restrict__ msg_base,
                                                            uint8_t *__restrict__ reach_base,
                                                            const int32_t *__restrict__ cur_node,
                                                            int write_reach)
{
    extern __shared__ float lds[];
    const int H = mv.H, L = mv.L;
    const int b = blockIdx.x, dir = blockIdx.y, tid = threadIdx.x;
    float *buf_a = lds, *buf_b = lds + kTile * H;
    float *msg = msg_base + static_cast<size_t>(dir) * gv.n_tot * H;
    uint8_t *reach = reach_base + static_cast<size_t>(dir) * gv.n_tot;
    const int32_t *order = gv.order[dir];
    const int32_t *nbr_ptr = gv.nbr_ptr[dir], *nbr_idx = gv.nbr_idx[dir];
    const int32_t *lvl = gv.lvl_ptr[dir] + gv.lvl_off[b];
    const int depth = gv.lvl_off[b + 1] - gv.lvl_off[b] - 1;
    const int n_b = gv.node_off[b + 1] - gv.node_off[b];
    const int cur_local = cur_node[b];
    const int cur = (cur_local >= 0 && cur_local < n_b) ? gv.node_off[b] + cur_local : -1;
    const MlpRef &fn = mv.f[dir], &gn = mv.g[dir];

    for (int level = 0; level < depth; ++level) {
        const int beg = lvl[level], end = lvl[level + 1];
        for (int t0 = beg; t0 < end; t0 += kTile) {
            const int rows = min(kTile, end - t0);
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                const int v = order[t0 + r];
                float a = 0.0f;
                for (int p = nbr_ptr[v]; p < nbr_ptr[v + 1]; ++p)
                    a += msg[static_cast<size_t>(nbr_idx[p]) * H + h];
                buf_a[i] = a;
            }
            if (write_reach && tid < rows) {
                const int v = order[t0 + tid];
                int bit = 0;
                for (int p = nbr_ptr[v]; p < nbr_ptr[v + 1]; ++p) {
                    const int u = nbr_idx[p];
                    bit |= (u == cur) | reach[u];
                }
                reach[v] = static_cast<uint8_t>(bit);
            }
            __syncthreads();
            float *in = buf_a, *out = buf_b;
            for (int l = 0; l < L; ++l) {
                dense_layer<RPT>(mv.blob + gn.layer[l].w, mv.blob + gn.layer[l].b, H, H, in, H,
                                 out, H, rows, true);
                __syncthreads();
                float *t = in; in = out; out = t;
            }
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                const size_t at = static_cast<size_t>(order[t0 + r]) * 2 * H + dir * H + h;
                const float s = emb[at] + in[i];
                emb[at] = s;
                in[i] = s;
            }
            __syncthreads();
            for (int l = 0; l < L; ++l) {
                dense_layer<RPT>(mv.blob + fn.layer[l].w, mv.blob + fn.layer[l].b, H, H, in, H,
                                 out, H, rows, true);
                __syncthreads();
                float *t = in; in = out; out = t;
            }
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                msg[static_cast<size_t>(order[t0 + r]) * H + h] = in[i];
            }
            __syncthreads();
        }
        // messages of this level are read by later levels of this same workgroup
        __threadfence_block();
        __syncthreads();
    }
}

// The reachability bits alone (k = 0 sweeps, or when only the node sets are wanted).
__global__ __launch_bounds__(kThreads) void k_reach_only(GraphView gv,
                                                         const int32_t *__restrict__ cur_node,
                                                         uint8_t *__restrict__ reach_base)
{
    const int b = blockIdx.x, dir = blockIdx.y, tid = threadIdx.x;
    uint8_t *reach = reach_base + static_cast<size_t>(dir) * gv.n_tot;
    const int32_t *order = gv.order[dir];
    const int32_t *nbr_ptr = gv.nbr_ptr[dir], *nbr_idx = gv.nbr_idx[dir];
    const int32_t *lvl = gv.lvl_ptr[dir] + gv.lvl_off[b];
    const int depth = gv.lvl_off[b + 1] - gv.lvl_off[b] - 1;
    const int n_b = gv.node_off[b + 1] - gv.node_off[b];
    const int cur_local = cur_node[b];
    const int cur = (cur_local >= 0 && cur_local < n_b) ? gv.node_off[b] + cur_local : -1;
    for (int level = 0; level < depth; ++level) {
        for (int t = lvl[level] + tid; t < lvl[level + 1]; t += kThreads) {
            const int v = order[t];
            int bit = 0;
            for (int p = nbr_ptr[v]; p < nbr_ptr[v + 1]; ++p) {
                const int u = nbr_idx[p];
                bit |= (u == cur) | reach[u];
            }
            reach[v] = static_cast<uint8_t>(bit);
        }
        __threadfence_block();
        __syncthreads();
    }
}

// The same for graphs whose lists fit in LDS: one wave per (graph, direction) copies the graph's
// bucket order, neighbour lists (graph-local ids) and level bounds into LDS and walks the levels
// there; a level then costs a chain of LDS reads instead of a chain of global loads.
__global__ __launch_bounds__(64) void k_reach_lds(GraphView gv, const int32_t *__restrict__ cur_node,
                                                  uint8_t *__restrict__ reach_base, int n_max, int e_max,
                                                  int depth_max)
{
    extern __shared__ int32_t reach_sm[];
    int32_t *s_order = reach_sm;                    // [n_max]     local ids in bucket order
    int32_t *s_ptr = s_order + n_max;               // [n_max + 1] local offsets of the neighbour lists
    int32_t *s_idx = s_ptr + n_max + 1;             // [e_max]     local neighbour ids
    int32_t *s_lvl = s_idx + e_max;                 // [depth_max + 1] local bucket bounds
    uint8_t *s_bit = reinterpret_cast<uint8_t *>(s_lvl + depth_max + 1);   // [n_max]
    const int b = blockIdx.x, dir = blockIdx.y, lane = threadIdx.x;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int32_t *nbr_ptr = gv.nbr_ptr[dir] + n0;
    const int e0 = nbr_ptr[0], e_b = nbr_ptr[n_b] - e0;
    const int32_t *lvl = gv.lvl_ptr[dir] + gv.lvl_off[b];
    const int depth = gv.lvl_off[b + 1] - gv.lvl_off[b] - 1;
    const int cur_local = cur_node[b];
    const int cur = (cur_local >= 0 && cur_local < n_b) ? cur_local : -1;
    for (int i = lane; i < n_b; i += 64) {
        s_order[i] = gv.order[dir][n0 + i] - n0;
        s_bit[i] = 0;
    }
    for (int i = lane; i <= n_b; i += 64) s_ptr[i] = nbr_ptr[i] - e0;
    for (int i = lane; i < e_b; i += 64) s_idx[i] = gv.nbr_idx[dir][e0 + i] - n0;
    for (int i = lane; i <= depth; i += 64) s_lvl[i] = lvl[i] - n0;
    __syncthreads();
    for (int level = 0; level < depth; ++level) {
        for (int t = s_lvl[level] + lane; t < s_lvl[level + 1]; t += 64) {
            const int v = s_order[t];
            int bit = 0;
            for (int p = s_ptr[v]; p < s_ptr[v + 1]; ++p) {
                const int u = s_idx[p];
                bit |= (u == cur) | s_bit[u];
            }
            s_bit[v] = static_cast<uint8_t>(bit);
        }
        __syncthreads();
    }
    uint8_t *reach = reach_base + static_cast<size_t>(dir) * gv.n_tot + n0;
    for (int i = lane; i < n_b; i += 64) reach[i] = s_bit[i];
}

// Section 2.2 step 3: 0 = v*, 1 = can reach v*, 2 = reachable from v*, 3 = neither.
// With `single` every node other than v* counts as a member of the first set.
__device__ __forceinline__ int node_class(int v, int cur, const uint8_t *reach, int n_tot, int single = 0)
{
    if (v == cur) return 0;
    if (single) return 1;
    if (reach[static_cast<size_t>(n_tot) + v]) return 1;   // bottom-up bit: ancestor of v*
    if (reach[v]) return 2;                                // top-down bit: descendant of v*
    return 3;
}

__global__ __launch_bounds__(kThreads) void k_classes(GraphView gv,
                                                      const int32_t *__restrict__ cur_node,
                                                      const uint8_t *__restrict__ reach,
                                                      uint8_t *__restrict__ out_class)
{
    const int v = blockIdx.x * kThreads + threadIdx.x;
    if (v >= gv.n_tot) return;
    const int b = gv.node_graph[v];
    const int n_b = gv.node_off[b + 1] - gv.node_off[b];
    const int c = cur_node[b];
    const int cur = (c >= 0 && c < n_b) ? gv.node_off[b] + c : -1;
    out_class[v] = static_cast<uint8_t>(node_class(v, cur, reach, gv.n_tot));
}

// ------------------------------------------------------------------ step 3: pooling
// Workgroup (chunk c, graph b) handles a contiguous slice of the graph's nodes.  Nodes are
// bucketed by set (in node order, so the summation order is fixed), pushed through that
// set's l network in tiles, and summed per (set, device group) into LDS accumulators.
// Partial sums go to partial[b][c][3G][H]; the head kernel adds the chunks in order.
constexpr int kSub = 256;   // nodes classified at a time

template <int RPT>
__global__ __launch_bounds__(kThreads) void k_pool_generic(GraphView gv, ModelView mv,
                                                           const float *__restrict__ emb,
                                                           const uint8_t *__restrict__ reach,
                                                           const int32_t *__restrict__ placement,
                                                           const int32_t *__restrict__ cur_node,
                                                           float *__restrict__ partial,
                                                           int max_chunks)
{
    extern __shared__ float lds[];
    __shared__ int16_t s_list[3][kSub];
    __shared__ int8_t s_cls[kSub];
    __shared__ int s_count[3];
    __shared__ int s_dev[kTile];
    const int H = mv.H, G = mv.G, D = mv.D, L = mv.L;
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    int chunks = (n_b + kPoolChunk - 1) / kPoolChunk;
    if (chunks > max_chunks) chunks = max_chunks;
    if (c >= chunks) return;
    const int per = (n_b + chunks - 1) / chunks;
    const int lo = n0 + c * per, hi = min(n0 + n_b, lo + per);
    const int cl = cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;

    float *acc = lds;                       // [3G][H]
    float *buf_x = acc + 3 * G * H;         // [kTile][2H]
    float *buf_a = buf_x + kTile * 2 * H;   // [kTile][H]
    float *buf_b = buf_a + kTile * H;       // [kTile][H]
    for (int i = tid; i < 3 * G * H; i += kThreads) acc[i] = 0.0f;

    for (int s0 = lo; s0 < hi; s0 += kSub) {
        const int cnt = min(kSub, hi - s0);
        if (tid < cnt) s_cls[tid] = static_cast<int8_t>(node_class(s0 + tid, cur, reach, gv.n_tot, mv.single_set));
        __syncthreads();
        if (tid < 3) {
            int m = 0;
            for (int i = 0; i < cnt; ++i)
                if (s_cls[i] == tid + 1) s_list[tid][m++] = static_cast<int16_t>(i);
            s_count[tid] = m;
        }
        __syncthreads();
        for (int set = 0; set < 3; ++set) {
            const int m = s_count[set];
            const MlpRef &ln = mv.l[set];
            for (int t0 = 0; t0 < m; t0 += kTile) {
                const int rows = min(kTile, m - t0);
                for (int i = tid; i < rows * 2 * H; i += kThreads) {
                    const int r = i / (2 * H), k = i - r * 2 * H;
                    buf_x[i] = emb[static_cast<size_t>(s0 + s_list[set][t0 + r]) * 2 * H + k];
                }
                if (tid < rows) {
                    const int dev = placement[s0 + s_list[set][t0 + tid]];
                    s_dev[tid] = (dev >= 0 && dev < D) ? (G == 1 ? 0 : dev) : -1;
                }
                __syncthreads();
                const float *in = buf_x;
                int n_in = 2 * H;
                float *out = buf_a;
                for (int l = 0; l < L; ++l) {
                    dense_layer<RPT>(mv.blob + ln.layer[l].w, mv.blob + ln.layer[l].b, n_in, H, in,
                                     n_in, out, H, rows, true);
                    __syncthreads();
                    in = out;
                    n_in = H;
                    out = (out == buf_a) ? buf_b : buf_a;
                }
                if (tid < H) {
                    for (int r = 0; r < rows; ++r) {
                        const int dev = s_dev[r];
                        if (dev >= 0) acc[(set * G + dev) * H + tid] += in[r * H + tid];
                    }
                }
                __syncthreads();
            }
        }
    }
    float *dst = partial + (static_cast<size_t>(b) * max_chunks + c) * 3 * G * H;
    for (int i = tid; i < 3 * G * H; i += kThreads) dst[i] = acc[i];
}

// ------------------------------------------------------------------ policy head
// Three small kernels, parallel over (graph, set), over (16 graphs, slice of Z) and over
// graphs: q[i][d] = h_i(P[i][d]) (also for empty groups); z = [e_{v*} ; q]; two-layer policy
// network with a softmax over devices (Appendix A.7).
constexpr int kZSlice = 256;   // inputs of policy layer 1 handled by one workgroup

// (1) workgroup (set, graph): P[set] = sum of the pooling partials in slice order, then h_set;
// set 0 also copies the current node's own embedding into z.
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_head_sets(GraphView gv, ModelView mv,
                                                        const float *__restrict__ emb,
                                                        const float *__restrict__ partial,
                                                        const int32_t *__restrict__ cur_node,
                                                        int max_chunks, float *__restrict__ zbuf,
                                                        float *__restrict__ out_pooled)
{
    extern __shared__ float lds[];
    const int H = mv.H, G = mv.G, L = mv.L, Z = mv.Z;
    const int set = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    int chunks = (n_b + kPoolChunk - 1) / kPoolChunk;
    if (chunks > max_chunks) chunks = max_chunks;
    float *P = lds;                     // [G][H]
    float *buf_a = P + kTile * H;       // [kTile][H]
    float *buf_b = buf_a + kTile * H;
    float *z = zbuf + static_cast<size_t>(b) * Z;
    const float *src = partial + (static_cast<size_t>(b) * max_chunks * 3 + set) * G * H;
    for (int i = tid; i < G * H; i += kThreads) {
        float s = 0.0f;
        for (int c = 0; c < chunks; ++c) s += src[static_cast<size_t>(c) * 3 * G * H + i];
        P[i] = s;
        if (out_pooled) out_pooled[(static_cast<size_t>(b) * 3 + set) * G * H + i] = s;
    }
    if (set == 0) {
        const int cl = cur_node[b];
        const bool ok = cl >= 0 && cl < n_b;
        for (int i = tid; i < 2 * H; i += kThreads)
            z[i] = ok ? emb[static_cast<size_t>(n0 + cl) * 2 * H + i] : 0.0f;
    }
    __syncthreads();
    const MlpRef &hn = mv.h[set];
    const float *in = P;
    for (int l = 0; l < L; ++l) {
        float *out = (l & 1) ? buf_b : buf_a;
        dense_layer<RPT, true>(mv.blob + hn.layer[l].w, mv.blob + hn.layer[l].b, H, H, in, H, out, H, G, true);
        __syncthreads();
        in = out;
    }
    for (int i = tid; i < G * H; i += kThreads) z[(2 + set * G) * H + i] = in[i];
}

// (2) workgroup (row tile, slice): partial products of policy layer 1 for 16 graphs and one
// slice of z: hidp[slice][b][j] = sum over k in the slice of z[b][k] W1[k][j].
// The two policy layers accumulate in float64 (the first one in blocks of sixteen fp32 terms):
// z holds sums over thousands of nodes, so a logit is a difference of terms far larger than
// itself, and a running fp32 sum over the (2 + 3G) H inputs alone would cost about 1e-6 of the
// largest logit of the graph, several times what the rest of the pass contributes.
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_head_policy1(ModelView mv, int B,
                                                           const float *__restrict__ zbuf,
                                                           double *__restrict__ hidp)
{
    __shared__ float x[kTile][kZSlice];
    const int H = mv.H, Z = mv.Z, tid = threadIdx.x;
    const int b0 = blockIdx.x * kTile, slice = blockIdx.y;
    const int k0 = slice * kZSlice, kn = min(kZSlice, Z - k0);
    const int rows = min(kTile, B - b0);
    for (int i = tid; i < rows * kZSlice; i += kThreads) {
        const int r = i / kZSlice, k = i - r * kZSlice;
        x[r][k] = k < kn ? zbuf[static_cast<size_t>(b0 + r) * Z + k0 + k] : 0.0f;
    }
    __syncthreads();
    // same thread mapping as dense_layer, without bias and activation
    int groups = kThreads / H;
    if (groups > kTile) groups = kTile;
    const int grp = tid / H, j = tid - grp * H;
    if (grp >= groups || grp >= rows) return;
    double acc[RPT];
    int xoff[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        acc[i] = 0.0;
        xoff[i] = min(grp + i * groups, rows - 1) * kZSlice;
    }
    const float *W = mv.blob + mv.pol1.w + static_cast<size_t>(k0) * H;
    const float *xf = &x[0][0];
    // terms per float64 block; weights per batch of loads, in flight together (the deeper batch pays
    // where a thread takes eight rows: 41 -> 35 us at H = 128; with four rows it cost 14 -> 24 us)
    constexpr int KB = 16, KL = RPT >= 8 ? 64 : 16;
    int k = 0;
    // sixteen terms in fp32, the blocks in float64: rounding errors stay relative to a
    // block's own size instead of the running sum's
    auto block = [&](const float *w, int kk) __attribute__((always_inline)) {
        float part[RPT];
#pragma unroll
        for (int i = 0; i < RPT; ++i) part[i] = 0.0f;
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int i = 0; i < RPT; ++i) part[i] = fmaf(xf[xoff[i] + kk + u], w[u], part[i]);
#pragma unroll
        for (int i = 0; i < RPT; ++i) acc[i] += static_cast<double>(part[i]);
    };
    for (; k + KL <= kn; k += KL) {
        float w[KL];
#pragma unroll
        for (int u = 0; u < KL; ++u) w[u] = W[static_cast<size_t>(k + u) * H + j];
#pragma unroll
        for (int u0 = 0; u0 < KL; u0 += KB) block(w + u0, k + u0);
    }
    for (; k + KB <= kn; k += KB) {
        float w[KB];
#pragma unroll
        for (int u = 0; u < KB; ++u) w[u] = W[static_cast<size_t>(k + u) * H + j];
        block(w, k);
    }
    for (; k < kn; ++k) {
        const double w = static_cast<double>(W[static_cast<size_t>(k) * H + j]);
#pragma unroll
        for (int i = 0; i < RPT; ++i) acc[i] = fma(static_cast<double>(xf[xoff[i] + k]), w, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = grp + i * groups;
        if (r < rows) hidp[(static_cast<size_t>(slice) * B + b0 + r) * H + j] = acc[i];
    }
}

// (3) one workgroup per graph: hidden = relu(sum of the slices + bias), output layer, softmax.
// policy_hidden / policy_logit (internal.h) are shared with the reverse pass, which forms the same
// logits again and must get the same bits.
__global__ __launch_bounds__(64) void k_head_out(GraphView gv, ModelView mv,
                                                 const double *__restrict__ hidp, int n_slices,
                                                 const int32_t *__restrict__ cur_node,
                                                 float *__restrict__ out_logits,
                                                 float *__restrict__ out_probs)
{
    __shared__ double hid[kMaxH];
    __shared__ float logit[kMaxD];
    const int H = mv.H, D = mv.D, b = blockIdx.x, tid = threadIdx.x;
    const int n_b = gv.node_off[b + 1] - gv.node_off[b];
    const int cl = cur_node[b];
    const bool cur_ok = cl >= 0 && cl < n_b;
    for (int j = tid; j < H; j += 64) hid[j] = policy_hidden(mv, hidp, n_slices, gv.B, b, j);
    __syncthreads();
    if (tid < D) logit[tid] = policy_logit(mv, hid, tid);
    __syncthreads();
    if (tid == 0) {
        float mx = logit[0];
        for (int d = 1; d < D; ++d) mx = fmaxf(mx, logit[d]);
        float tot = 0.0f;
        for (int d = 0; d < D; ++d) tot += expf(logit[d] - mx);
        const float bad = __builtin_nanf("");   // no valid current node: nothing to decide
        for (int d = 0; d < D; ++d) {
            out_logits[static_cast<size_t>(b) * D + d] = cur_ok ? logit[d] : bad;
            if (out_probs) out_probs[static_cast<size_t>(b) * D + d] = cur_ok ? expf(logit[d] - mx) / tot : bad;
        }
    }
}

int pick_rpt(int H)
{
    int groups = kThreads / H;
    if (groups > kTile) groups = kTile;
    int rpt = 1;
    while (groups * rpt < kTile) rpt *= 2;
    return rpt;
}

template <typename K>
void allow_lds(K kernel, size_t bytes)
{
    if (bytes > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize,
                                  static_cast<int>(bytes));
}

#define PL_DISPATCH_RPT(rpt, CALL) \
    switch (rpt) {                 \
        case 1: { CALL(1); break; }  \
        case 2: { CALL(2); break; }  \
        case 4: { CALL(4); break; }  \
        case 8: { CALL(8); break; }  \
        default: { CALL(16); break; } \
    }

}  // namespace

void launch_project(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                    const ForwardArgs &fa, bool to_emb, bool to_xb, hipStream_t s)
{
    const size_t total = static_cast<size_t>(gv.n_tot) * mv.H;
    if (total == 0) return;
    if (mv.H % 4 == 0) {
        const unsigned blocks = static_cast<unsigned>((total / 4 + kThreads - 1) / kThreads);
        hipLaunchKernelGGL(k_project4, dim3(blocks), dim3(kThreads), 0, s, gv, mv, fa.node_feats,
                           fa.placement, fa.cur_node, to_emb ? ws.emb : nullptr, to_xb ? ws.xb : nullptr);
        return;
    }
    const unsigned blocks = static_cast<unsigned>((total + kThreads - 1) / kThreads);
    hipLaunchKernelGGL(k_project, dim3(blocks), dim3(kThreads), 0, s, gv, mv, fa.node_feats,
                       fa.placement, fa.cur_node, to_emb ? ws.emb : nullptr, to_xb ? ws.xb : nullptr);
}

void launch_sweep_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                          const ForwardArgs &fa, bool write_reach, hipStream_t s)
{
    if (gv.B == 0) return;
    const size_t lds = sizeof(float) * 2 * kTile * mv.H;
#define CALL(R)                                                                               \
    allow_lds(k_sweep_generic<R>, lds);                                                       \
    hipLaunchKernelGGL(k_sweep_generic<R>, dim3(gv.B, 2), dim3(kThreads), lds, s, gv, mv, ws.emb, \
                       ws.msg, ws.reach, fa.cur_node, write_reach ? 1 : 0)
    PL_DISPATCH_RPT(pick_rpt(mv.H), CALL)
#undef CALL
}

void launch_reach_only(const GraphView &gv, const int32_t *cur_node, uint8_t *reach, int n_max, int e_max,
                       int depth_max, hipStream_t s)
{
    if (gv.B == 0) return;
    // largest graph's order, list offsets, lists, level bounds and bits
    const size_t lds = sizeof(int32_t) * (2 * static_cast<size_t>(n_max) + 1 + e_max + depth_max + 1) + n_max;
    if (n_max > 0 && lds <= 64 * 1024) {
        allow_lds(k_reach_lds, lds);
        hipLaunchKernelGGL(k_reach_lds, dim3(gv.B, 2), dim3(64), lds, s, gv, cur_node, reach, n_max, e_max, depth_max);
        return;
    }
    hipLaunchKernelGGL(k_reach_only, dim3(gv.B, 2), dim3(kThreads), 0, s, gv, cur_node, reach);
}

void launch_classes(const GraphView &gv, const int32_t *cur_node, const uint8_t *reach,
                    uint8_t *out_class, hipStream_t s)
{
    if (gv.n_tot == 0) return;
    hipLaunchKernelGGL(k_classes, dim3((gv.n_tot + kThreads - 1) / kThreads), dim3(kThreads), 0, s,
                       gv, cur_node, reach, out_class);
}

void launch_pool_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                         const ForwardArgs &fa, hipStream_t s)
{
    if (gv.B == 0) return;
    const size_t lds = sizeof(float) * (static_cast<size_t>(3) * mv.G * mv.H + kTile * 4 * mv.H);
#define CALL(R)                                                                              \
    allow_lds(k_pool_generic<R>, lds);                                                       \
    hipLaunchKernelGGL(k_pool_generic<R>, dim3(ws.n_chunks, gv.B), dim3(kThreads), lds, s, gv, mv, \
                       ws.emb, ws.reach, fa.placement, fa.cur_node, ws.partial, ws.n_chunks)
    PL_DISPATCH_RPT(pick_rpt(mv.H), CALL)
#undef CALL
}

void launch_head_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                         const ForwardArgs &fa, int max_chunks, hipStream_t s)
{
    if (gv.B == 0) return;
    const size_t lds = sizeof(float) * 3 * kTile * mv.H;
    const int n_slices = (mv.Z + kZSlice - 1) / kZSlice;
    const int row_tiles = (gv.B + kTile - 1) / kTile;
    // h_i works on the G rows of a set, the first policy layer on tiles of kTile graphs: each
    // thread takes as many rows as that needs
    int groups = kThreads / mv.H;
    if (groups > kTile) groups = kTile;
    if (groups < 1) groups = 1;
    int rpt_sets = 1;
    while (groups * rpt_sets < mv.G) rpt_sets *= 2;
#define CALL(R)                                                                                  \
    hipLaunchKernelGGL(k_head_sets<R>, dim3(3, gv.B), dim3(kThreads), lds, s, gv, mv, ws.emb,    \
                       ws.partial, fa.cur_node, max_chunks, ws.zbuf, fa.out_pooled)
    PL_DISPATCH_RPT(rpt_sets, CALL)
#undef CALL
#define CALL(R)                                                                                  \
    hipLaunchKernelGGL(k_head_policy1<R>, dim3(row_tiles, n_slices), dim3(kThreads), 0, s, mv,   \
                       gv.B, ws.zbuf, ws.hidp)
    PL_DISPATCH_RPT(pick_rpt(mv.H), CALL)
#undef CALL
    hipLaunchKernelGGL(k_head_out, dim3(gv.B), dim3(64), 0, s, gv, mv, ws.hidp, n_slices, fa.cur_node,
                       fa.out_logits, fa.out_probs);
}

}  // namespace pl
