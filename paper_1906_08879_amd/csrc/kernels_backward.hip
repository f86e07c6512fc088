// Reverse-mode pass of the policy network: the gradient of log pi(a | s) with respect to every
// parameter, summed over a batch with one scalar per state.  This is the term
// grad_theta log pi_theta(a_i | s_i) * (return - baseline) of the REINFORCE update (appendix
// "REINFORCE Algorithm", Eq. 1) for the network of Section 2.2 / Appendix A.7.
//
// The forward pass leaves the node embeddings e_v = [td_v ; bu_v], the pooled sums and the
// policy inputs in the batch's buffers.  From them:
//   1. head:   d logits = c (one-hot(a) - pi); back through the policy layers and h_i to the
//              pooled sums P[i][d] and to e_{v*};
//   2. pool:   every node u of set i on device d receives dP[i][d]; back through l_i to e_u;
//   3. sweeps: activations of f and g are recomputed for all nodes at once (they depend only
//              on the final states), then one workgroup per (graph, direction) walks the levels
//              in REVERSE order: a node's state gradient needs the gradients of all the sums it
//              was gathered into, which belong to later levels;
//   4. projection: both directions start from x_v, so its gradient is the sum of the two;
//   5. every weight gradient is a contraction over rows (nodes, pooled groups or graphs) of
//              layer input x layer delta, done in slabs with a fixed summation order (no
//              atomics).
// Two sets of kernels: generic fp32 vector kernels for any H <= 256, D <= 16, 1..4 layers; and,
// for H in {32, 64, 128}, the parallel parts (per-node layers, weight gradients) on the fp32
// matrix cores (v_mfma_f32_32x32x2_f32) and the dependent chain of step 3 in the matrix-core sweep
// kernel run in reverse.  Several sweeps are differentiated from the last to the first.
#include <algorithm>

#include "internal.h"

namespace pl {

namespace {

constexpr int kThreads = 256;
constexpr int kTile = 16;      // rows pushed through a layer together
constexpr int kWgI = 16;       // weight-matrix rows per workgroup of the contraction kernel
constexpr int kWgRB = 32;      // contraction rows staged at a time
constexpr int kPoolSub = 256;  // nodes classified at a time

// y[r][j] = bias[j] + sum_k x[r][k] * W[k * ldw + j] for r < rows (<= kTile), j < n_out, optional
// ReLU.  x and y in LDS.  Thread (grp, j) owns rows grp, grp + groups, ...  Requires
// n_out <= kThreads and min(kThreads / n_out, kTile) * RPT >= rows.  bias may be null.
template <int RPT>
__device__ __forceinline__ void dense_rows(const float *__restrict__ W, int ldw,
                                           const float *__restrict__ bias, int n_in, int n_out,
                                           const float *x, int ldx, float *y, int ldy, int rows,
                                           bool relu)
{
    const int tid = threadIdx.x;
    int groups = kThreads / n_out;
    if (groups > kTile) groups = kTile;
    const int grp = tid / n_out, j = tid - grp * n_out;
    if (grp >= groups || grp >= rows) return;
    float acc[RPT];
    const float bj = bias ? bias[j] : 0.0f;
#pragma unroll
    for (int i = 0; i < RPT; ++i) acc[i] = bj;
    int xoff[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) xoff[i] = min(grp + i * groups, rows - 1) * ldx;
    constexpr int KB = 16;
    int k = 0;
    for (; k + KB <= n_in; k += KB) {
        float w[KB];
#pragma unroll
        for (int u = 0; u < KB; ++u) w[u] = W[static_cast<size_t>(k + u) * ldw + j];
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int i = 0; i < RPT; ++i) acc[i] = fmaf(x[xoff[i] + k + u], w[u], acc[i]);
    }
    for (; k < n_in; ++k) {
        const float w = W[static_cast<size_t>(k) * ldw + j];
#pragma unroll
        for (int i = 0; i < RPT; ++i) acc[i] = fmaf(x[xoff[i] + k], w, acc[i]);
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const int r = grp + i * groups;
        if (r < rows) y[r * ldy + j] = relu ? fmaxf(acc[i], 0.0f) : acc[i];
    }
}

// Position of activation / delta array (dir, layer) inside a [2][L][n_tot][H] buffer.
__device__ __forceinline__ size_t slab(int dir, int l, int L, int n_tot, int H)
{
    return (static_cast<size_t>(dir) * L + l) * static_cast<size_t>(n_tot) * H;
}

// ------------------------------------------------------------------ 1. policy head
// One workgroup per graph: logits again from the stored partial products of policy layer 1,
// d logits = c (one-hot(a) - softmax), back to the hidden layer and to the policy input z.
// A graph whose current node or action is out of range gets a zero gradient and logp = NaN.
__global__ __launch_bounds__(kThreads) void k_bw_head(GraphView gv, ModelView mv,
                                                      const float *__restrict__ blob_t,
                                                      const double *__restrict__ hidp, int n_slices,
                                                      const int32_t *__restrict__ cur_node,
                                                      const int32_t *__restrict__ actions,
                                                      const float *__restrict__ coeff,
                                                      const float *__restrict__ ent_coeff,
                                                      float *__restrict__ out_entropy,
                                                      float *__restrict__ hid_out,
                                                      float *__restrict__ dpre_out,
                                                      float *__restrict__ dlogit_out,
                                                      float *__restrict__ dz,
                                                      float *__restrict__ out_logp)
{
    __shared__ double hid64[kMaxH];
    __shared__ float hid[kMaxH];
    __shared__ float dpre[kMaxH];
    __shared__ float logit[kMaxD];
    __shared__ float dlog[kMaxD];
    const int H = mv.H, D = mv.D, b = blockIdx.x, tid = threadIdx.x;
    const int n_b = gv.node_off[b + 1] - gv.node_off[b];
    const int cl = cur_node[b];
    const bool cur_ok = cl >= 0 && cl < n_b;
    for (int j = tid; j < H; j += kThreads) {
        hid64[j] = policy_hidden(mv, hidp, n_slices, gv.B, b, j);
        hid[j] = static_cast<float>(hid64[j]);
    }
    __syncthreads();
    if (tid < D) logit[tid] = policy_logit(mv, hid64, tid);
    __syncthreads();
    if (tid == 0) {
        float mx = logit[0];
        for (int d = 1; d < D; ++d) mx = fmaxf(mx, logit[d]);
        float tot = 0.0f;
        for (int d = 0; d < D; ++d) tot += expf(logit[d] - mx);
        const int a = actions[b];
        const bool ok = cur_ok && a >= 0 && a < D;
        const float c = ok ? coeff[b] : 0.0f;
        // entropy term (Appendix A.7): H = - sum p log p, dH / d logit_d = - p_d (log p_d + H), with
        // log p_d = logit_d - max - log(sum), which stays finite where p_d underflows to 0
        const float beta = (ok && ent_coeff) ? ent_coeff[b] : 0.0f;
        const float lse = logf(tot);
        float ent = 0.0f;
        for (int d = 0; d < D; ++d) {
            const float p = expf(logit[d] - mx) / tot;
            ent -= p * ((logit[d] - mx) - lse);
        }
        for (int d = 0; d < D; ++d) {
            const float p = expf(logit[d] - mx) / tot;
            dlog[d] = c * ((d == a ? 1.0f : 0.0f) - p) - beta * p * (((logit[d] - mx) - lse) + ent);
        }
        if (out_logp) out_logp[b] = ok ? (logit[a] - mx) - lse : __builtin_nanf("");
        if (out_entropy) out_entropy[b] = cur_ok ? ent : __builtin_nanf("");
    }
    __syncthreads();
    for (int j = tid; j < H; j += kThreads) {
        const float *W = mv.blob + mv.pol2.w + static_cast<size_t>(j) * D;
        float s = 0.0f;
        for (int d = 0; d < D; ++d) s = fmaf(W[d], dlog[d], s);
        const float dp = hid[j] > 0.0f ? s : 0.0f;
        dpre[j] = dp;
        hid_out[static_cast<size_t>(b) * H + j] = hid[j];
        dpre_out[static_cast<size_t>(b) * H + j] = dp;
    }
    if (tid < D) dlogit_out[static_cast<size_t>(b) * D + tid] = dlog[tid];
}

// dz[b][k] = sum_j W1[k][j] dpre[b][j] for kDzGraphs graphs per workgroup and one 256-wide slice of
// the policy input: a weight is loaded once for all the workgroup's graphs (one workgroup per graph
// read the whole first policy layer, 1.7 MB at the NASNet-like shape, from L2 every time).
constexpr int kDzGraphs = 8;
__global__ __launch_bounds__(kThreads) void k_bw_dz(ModelView mv, int B, const float *__restrict__ blob_t,
                                                    const float *__restrict__ dpre, float *__restrict__ dz)
{
    __shared__ float dp[kDzGraphs][kMaxH];
    const int H = mv.H, Z = mv.Z, tid = threadIdx.x;
    const int k = blockIdx.x * kThreads + tid, b0 = blockIdx.y * kDzGraphs;
    const int nb = min(kDzGraphs, B - b0);
    for (int i = tid; i < kDzGraphs * H; i += kThreads) {
        const int g = i / H, j = i - g * H;
        dp[g][j] = g < nb ? dpre[static_cast<size_t>(b0 + g) * H + j] : 0.0f;
    }
    __syncthreads();
    if (k >= Z) return;
    const float *W1t = blob_t + mv.pol1.w;   // [H][Z]
    float acc[kDzGraphs];
#pragma unroll
    for (int g = 0; g < kDzGraphs; ++g) acc[g] = 0.0f;
    constexpr int KB = 16;                   // weights per batch of loads
    int j = 0;
    for (; j + KB <= H; j += KB) {
        float w[KB];
#pragma unroll
        for (int u = 0; u < KB; ++u) w[u] = W1t[static_cast<size_t>(j + u) * Z + k];
#pragma unroll
        for (int u = 0; u < KB; ++u)
#pragma unroll
            for (int g = 0; g < kDzGraphs; ++g) acc[g] = fmaf(w[u], dp[g][j + u], acc[g]);
    }
    for (; j < H; ++j) {
        const float w = W1t[static_cast<size_t>(j) * Z + k];
#pragma unroll
        for (int g = 0; g < kDzGraphs; ++g) acc[g] = fmaf(w, dp[g][j], acc[g]);
    }
#pragma unroll
    for (int g = 0; g < kDzGraphs; ++g)
        if (g < nb) dz[static_cast<size_t>(b0 + g) * Z + k] = acc[g];
}

// Workgroup (set, graph): q[set][d] = h_set(P[set][d]) again for the G device groups, keeping
// every layer's output, then back from dz to dP[set][d].
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_bw_head_sets(GraphView gv, ModelView mv,
                                                           const float *__restrict__ blob_t,
                                                           const float *__restrict__ pooled,
                                                           const float *__restrict__ dz,
                                                           float *__restrict__ hin,
                                                           float *__restrict__ hact,
                                                           float *__restrict__ dh,
                                                           float *__restrict__ dP)
{
    extern __shared__ float lds[];
    const int H = mv.H, G = mv.G, L = mv.L, Z = mv.Z;
    const int set = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const size_t BG = static_cast<size_t>(gv.B) * G;
    float *buf_p = lds, *buf_a = lds + kTile * H, *buf_b = buf_a + kTile * H;
    const float *src = pooled + (static_cast<size_t>(b) * 3 + set) * G * H;
    for (int i = tid; i < G * H; i += kThreads) {
        const float v = src[i];
        buf_p[i] = v;
        hin[(static_cast<size_t>(set) * BG + static_cast<size_t>(b) * G) * H + i] = v;
    }
    __syncthreads();
    const MlpRef &hn = mv.h[set];
    const float *in = buf_p;
    for (int l = 0; l < L; ++l) {
        float *out = (l & 1) ? buf_b : buf_a;
        dense_rows<RPT>(mv.blob + hn.layer[l].w, H, mv.blob + hn.layer[l].b, H, H, in, H, out, H, G, true);
        __syncthreads();
        float *dst = hact + ((static_cast<size_t>(set) * L + l) * BG + static_cast<size_t>(b) * G) * H;
        for (int i = tid; i < G * H; i += kThreads) dst[i] = out[i];
        in = out;
    }
    __threadfence_block();
    __syncthreads();
    // delta of the last layer: dz of this set's slots, masked by the layer's output
    float *dcur = buf_a, *dnext = buf_b;
    {
        const float *act = hact + ((static_cast<size_t>(set) * L + (L - 1)) * BG + static_cast<size_t>(b) * G) * H;
        const float *g = dz + static_cast<size_t>(b) * Z + static_cast<size_t>(2 + set * G) * H;
        for (int i = tid; i < G * H; i += kThreads) dcur[i] = act[i] > 0.0f ? g[i] : 0.0f;
    }
    __syncthreads();
    for (int l = L - 1; l >= 0; --l) {
        float *dst = dh + ((static_cast<size_t>(set) * L + l) * BG + static_cast<size_t>(b) * G) * H;
        for (int i = tid; i < G * H; i += kThreads) dst[i] = dcur[i];
        dense_rows<RPT>(blob_t + hn.layer[l].w, H, nullptr, H, H, dcur, H, dnext, H, G, false);
        __syncthreads();
        if (l > 0) {
            const float *act = hact + ((static_cast<size_t>(set) * L + (l - 1)) * BG + static_cast<size_t>(b) * G) * H;
            for (int i = tid; i < G * H; i += kThreads) dnext[i] = act[i] > 0.0f ? dnext[i] : 0.0f;
        } else {
            float *out = dP + (static_cast<size_t>(b) * 3 + set) * G * H;
            for (int i = tid; i < G * H; i += kThreads) out[i] = dnext[i];
        }
        __syncthreads();
        float *t = dcur; dcur = dnext; dnext = t;
    }
}

// Section 2.2 step 3: 0 = v*, 1 = can reach v*, 2 = reachable from v*, 3 = neither.
__device__ __forceinline__ int node_class_bw(int v, int cur, const uint8_t *reach, int n_tot, int single)
{
    if (v == cur) return 0;
    if (single) return 1;                  // every node other than v* is in the first set
    if (reach[static_cast<size_t>(n_tot) + v]) return 1;
    if (reach[v]) return 2;
    return 3;
}

// ------------------------------------------------------------------ 2. pooling
// Workgroup (chunk, graph) over a contiguous slice of the graph's nodes, bucketed by set as in
// the forward pass.  A tile of nodes of one set goes forward through l_set (outputs kept in
// lact), takes dP[set][device] as the gradient of its last output, and goes back to d e_u.
// The current node takes its gradient from the policy input; a node with a device id outside
// [0, D) was pooled nowhere and gets zero.
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_bw_pool(GraphView gv, ModelView mv,
                                                      const float *__restrict__ blob_t,
                                                      const float *__restrict__ emb,
                                                      const uint8_t *__restrict__ reach,
                                                      const int32_t *__restrict__ placement,
                                                      const int32_t *__restrict__ cur_node,
                                                      const float *__restrict__ dP,
                                                      const float *__restrict__ dz,
                                                      uint8_t *__restrict__ cls_out,
                                                      float *__restrict__ lact,
                                                      float *__restrict__ dl,
                                                      float *__restrict__ demb, int max_chunks)
{
    extern __shared__ float lds[];
    __shared__ int16_t s_list[3][kPoolSub];
    __shared__ int8_t s_cls[kPoolSub];
    __shared__ int s_count[3];
    __shared__ int s_dev[kTile];
    __shared__ int s_node[kTile];
    const int H = mv.H, G = mv.G, D = mv.D, L = mv.L, Z = mv.Z;
    const int b = blockIdx.y, c = blockIdx.x, tid = threadIdx.x;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    int chunks = (n_b + kPoolChunk - 1) / kPoolChunk;
    if (chunks > max_chunks) chunks = max_chunks;
    if (c >= chunks) return;
    const int per = (n_b + chunks - 1) / chunks;
    const int lo = n0 + c * per, hi = min(n0 + n_b, lo + per);
    const int cl = cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    const size_t NH = static_cast<size_t>(gv.n_tot) * H;

    float *buf_x = lds;                    // [kTile][2H]
    float *buf_a = buf_x + kTile * 2 * H;  // [kTile][H]
    float *buf_b = buf_a + kTile * H;      // [kTile][H]

    for (int s0 = lo; s0 < hi; s0 += kPoolSub) {
        const int cnt = min(kPoolSub, hi - s0);
        if (tid < cnt) {
            const int k = node_class_bw(s0 + tid, cur, reach, gv.n_tot, mv.single_set);
            s_cls[tid] = static_cast<int8_t>(k);
            cls_out[s0 + tid] = static_cast<uint8_t>(k);
        }
        __syncthreads();
        if (tid < 3) {
            int m = 0;
            for (int i = 0; i < cnt; ++i)
                if (s_cls[i] == tid + 1) s_list[tid][m++] = static_cast<int16_t>(i);
            s_count[tid] = m;
        }
        // the current node: d e = first 2H entries of dz; its l rows are never used
        if (cur >= s0 && cur < s0 + cnt)
            for (int i = tid; i < 2 * H; i += kThreads)
                demb[static_cast<size_t>(cur) * 2 * H + i] = dz[static_cast<size_t>(b) * Z + i];
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
                    const int v = s0 + s_list[set][t0 + tid];
                    const int dev = placement[v];
                    s_node[tid] = v;
                    s_dev[tid] = (dev >= 0 && dev < D) ? (G == 1 ? 0 : dev) : -1;
                }
                __syncthreads();
                // forward through l_set, every layer's output kept
                const float *in = buf_x;
                int n_in = 2 * H;
                float *out = buf_a;
                for (int l = 0; l < L; ++l) {
                    dense_rows<RPT>(mv.blob + ln.layer[l].w, H, mv.blob + ln.layer[l].b, n_in, H, in, n_in,
                                    out, H, rows, true);
                    __syncthreads();
                    for (int i = tid; i < rows * H; i += kThreads) {
                        const int r = i / H, h = i - r * H;
                        lact[static_cast<size_t>(l) * NH + static_cast<size_t>(s_node[r]) * H + h] = out[i];
                    }
                    in = out;
                    n_in = H;
                    out = (out == buf_a) ? buf_b : buf_a;
                }
                // `in` holds the last layer's output; delta of the last layer into `out`
                float *dcur = out, *dnext = const_cast<float *>(in);
                for (int i = tid; i < rows * H; i += kThreads) {
                    const int r = i / H, h = i - r * H;
                    const int dev = s_dev[r];
                    const float g = dev >= 0 ? dP[((static_cast<size_t>(b) * 3 + set) * G + dev) * H + h] : 0.0f;
                    dcur[i] = in[i] > 0.0f ? g : 0.0f;
                }
                __threadfence_block();
                __syncthreads();
                for (int l = L - 1; l >= 0; --l) {
                    for (int i = tid; i < rows * H; i += kThreads) {
                        const int r = i / H, h = i - r * H;
                        dl[static_cast<size_t>(l) * NH + static_cast<size_t>(s_node[r]) * H + h] = dcur[i];
                    }
                    if (l > 0) {
                        dense_rows<RPT>(blob_t + ln.layer[l].w, H, nullptr, H, H, dcur, H, dnext, H, rows, false);
                        __syncthreads();
                        for (int i = tid; i < rows * H; i += kThreads) {
                            const int r = i / H, h = i - r * H;
                            const float a = lact[static_cast<size_t>(l - 1) * NH + static_cast<size_t>(s_node[r]) * H + h];
                            dnext[i] = a > 0.0f ? dnext[i] : 0.0f;
                        }
                        __syncthreads();
                        float *t = dcur; dcur = dnext; dnext = t;
                    } else {
                        // first layer: [2H, H] stored transposed as [H][2H]; the two halves of d e
                        dense_rows<RPT>(blob_t + ln.layer[0].w, 2 * H, nullptr, H, H, dcur, H, buf_x, 2 * H, rows, false);
                        dense_rows<RPT>(blob_t + ln.layer[0].w + H, 2 * H, nullptr, H, H, dcur, H, buf_x + H, 2 * H, rows, false);
                        __syncthreads();
                        for (int i = tid; i < rows * 2 * H; i += kThreads) {
                            const int r = i / (2 * H), k = i - r * 2 * H;
                            demb[static_cast<size_t>(s_node[r]) * 2 * H + k] = buf_x[i];
                        }
                    }
                }
                __syncthreads();
            }
        }
    }
}

// ------------------------------------------------------------------ 3. sweeps
// (a) f at the final state of every node: tile of 16 nodes x direction.
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_bw_f_acts(GraphView gv, ModelView mv,
                                                        const float *__restrict__ emb,
                                                        float *__restrict__ fact)
{
    extern __shared__ float lds[];
    const int H = mv.H, L = mv.L, tid = threadIdx.x, dir = blockIdx.y;
    const int v0 = blockIdx.x * kTile, rows = min(kTile, gv.n_tot - v0);
    float *buf_a = lds, *buf_b = lds + kTile * H;
    for (int i = tid; i < rows * H; i += kThreads) {
        const int r = i / H, h = i - r * H;
        buf_a[i] = emb[static_cast<size_t>(v0 + r) * 2 * H + dir * H + h];
    }
    __syncthreads();
    float *in = buf_a, *out = buf_b;
    for (int l = 0; l < L; ++l) {
        const LayerRef &ly = mv.f[dir].layer[l];
        dense_rows<RPT>(mv.blob + ly.w, H, mv.blob + ly.b, H, H, in, H, out, H, rows, true);
        __syncthreads();
        float *dst = fact + slab(dir, l, L, gv.n_tot, H) + static_cast<size_t>(v0) * H;
        for (int i = tid; i < rows * H; i += kThreads) dst[i] = out[i];
        float *t = in; in = out; out = t;
    }
}

// (b) the gathered sums a_v = sum of the neighbours' messages, and g at them.
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_bw_g_acts(GraphView gv, ModelView mv,
                                                        const float *__restrict__ fact,
                                                        float *__restrict__ agg,
                                                        float *__restrict__ gact)
{
    extern __shared__ float lds[];
    const int H = mv.H, L = mv.L, tid = threadIdx.x, dir = blockIdx.y;
    const int v0 = blockIdx.x * kTile, rows = min(kTile, gv.n_tot - v0);
    float *buf_a = lds, *buf_b = lds + kTile * H;
    const float *msg = fact + slab(dir, L - 1, L, gv.n_tot, H);
    const int32_t *nbr_ptr = gv.nbr_ptr[dir], *nbr_idx = gv.nbr_idx[dir];
    for (int i = tid; i < rows * H; i += kThreads) {
        const int r = i / H, h = i - r * H;
        const int v = v0 + r;
        float a = 0.0f;
        for (int p = nbr_ptr[v]; p < nbr_ptr[v + 1]; ++p) a += msg[static_cast<size_t>(nbr_idx[p]) * H + h];
        buf_a[i] = a;
        agg[(static_cast<size_t>(dir) * gv.n_tot + v) * H + h] = a;
    }
    __syncthreads();
    float *in = buf_a, *out = buf_b;
    for (int l = 0; l < L; ++l) {
        const LayerRef &ly = mv.g[dir].layer[l];
        dense_rows<RPT>(mv.blob + ly.w, H, mv.blob + ly.b, H, H, in, H, out, H, rows, true);
        __syncthreads();
        float *dst = gact + slab(dir, l, L, gv.n_tot, H) + static_cast<size_t>(v0) * H;
        for (int i = tid; i < rows * H; i += kThreads) dst[i] = out[i];
        float *t = in; in = out; out = t;
    }
}

// (c) the dependent chain.  s_v <- s_v + g(a_v), m_v = f(s_v), a_w = sum of m over xi(w).
// With dE/ds_v given from outside (pooling, head) in demb, for v in reverse level order:
//   dm_v   = sum over the nodes w that gathered m_v (v's neighbours in the OTHER direction) of da_w
//   ds_v  += f'(s_v)^T dm_v          (back through the layers of f)
//   da_v   = g'(a_v)^T ds_v          (back through the layers of g)
// demb becomes the gradient of the sweep's input (the residual passes ds_v through unchanged).
template <int RPT>
__global__ __launch_bounds__(kThreads) void k_bw_sweep_generic(GraphView gv, ModelView mv,
                                                               const float *__restrict__ blob_t,
                                                               const float *__restrict__ fact,
                                                               const float *__restrict__ gact,
                                                               float *__restrict__ demb,
                                                               float *__restrict__ dagg_base,
                                                               float *__restrict__ dfg, size_t dfg_stride)
{
    extern __shared__ float lds[];
    const int H = mv.H, L = mv.L;
    const int b = blockIdx.x, dir = blockIdx.y, tid = threadIdx.x;
    float *buf_a = lds, *buf_b = lds + kTile * H;
    float *dagg = dagg_base + static_cast<size_t>(dir) * gv.n_tot * H;
    const int32_t *order = gv.order[dir];
    const int32_t *suc_ptr = gv.nbr_ptr[1 - dir], *suc_idx = gv.nbr_idx[1 - dir];
    const int32_t *lvl = gv.lvl_ptr[dir] + gv.lvl_off[b];
    const int depth = gv.lvl_off[b + 1] - gv.lvl_off[b] - 1;
    const MlpRef &fn = mv.f[dir], &gn = mv.g[dir];
    const size_t NH = static_cast<size_t>(gv.n_tot) * H;
    float *df = dfg + dir * dfg_stride, *dg = df + L * NH;

    for (int level = depth - 1; level >= 0; --level) {
        const int beg = lvl[level], end = lvl[level + 1];
        for (int t0 = beg; t0 < end; t0 += kTile) {
            const int rows = min(kTile, end - t0);
            // dm_v, masked by the last layer of f
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                const int v = order[t0 + r];
                float a = 0.0f;
                for (int p = suc_ptr[v]; p < suc_ptr[v + 1]; ++p)
                    a += dagg[static_cast<size_t>(suc_idx[p]) * H + h];
                const float m = fact[slab(dir, L - 1, L, gv.n_tot, H) + static_cast<size_t>(v) * H + h];
                buf_a[i] = m > 0.0f ? a : 0.0f;
            }
            __syncthreads();
            float *dcur = buf_a, *dnext = buf_b;
            for (int l = L - 1; l >= 0; --l) {
                for (int i = tid; i < rows * H; i += kThreads) {
                    const int r = i / H, h = i - r * H;
                    df[l * NH + static_cast<size_t>(order[t0 + r]) * H + h] = dcur[i];
                }
                dense_rows<RPT>(blob_t + fn.layer[l].w, H, nullptr, H, H, dcur, H, dnext, H, rows, false);
                __syncthreads();
                if (l > 0) {
                    for (int i = tid; i < rows * H; i += kThreads) {
                        const int r = i / H, h = i - r * H;
                        const float a = fact[slab(dir, l - 1, L, gv.n_tot, H) + static_cast<size_t>(order[t0 + r]) * H + h];
                        dnext[i] = a > 0.0f ? dnext[i] : 0.0f;
                    }
                    __syncthreads();
                }
                float *t = dcur; dcur = dnext; dnext = t;
            }
            // ds_v = outside gradient + f-path; then the delta of g's last layer
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                const int v = order[t0 + r];
                const size_t at = static_cast<size_t>(v) * 2 * H + dir * H + h;
                const float ds = demb[at] + dcur[i];
                demb[at] = ds;
                const float u = gact[slab(dir, L - 1, L, gv.n_tot, H) + static_cast<size_t>(v) * H + h];
                dcur[i] = u > 0.0f ? ds : 0.0f;
            }
            __syncthreads();
            for (int l = L - 1; l >= 0; --l) {
                for (int i = tid; i < rows * H; i += kThreads) {
                    const int r = i / H, h = i - r * H;
                    dg[l * NH + static_cast<size_t>(order[t0 + r]) * H + h] = dcur[i];
                }
                dense_rows<RPT>(blob_t + gn.layer[l].w, H, nullptr, H, H, dcur, H, dnext, H, rows, false);
                __syncthreads();
                if (l > 0) {
                    for (int i = tid; i < rows * H; i += kThreads) {
                        const int r = i / H, h = i - r * H;
                        const float a = gact[slab(dir, l - 1, L, gv.n_tot, H) + static_cast<size_t>(order[t0 + r]) * H + h];
                        dnext[i] = a > 0.0f ? dnext[i] : 0.0f;
                    }
                    __syncthreads();
                }
                float *t = dcur; dcur = dnext; dnext = t;
            }
            for (int i = tid; i < rows * H; i += kThreads) {
                const int r = i / H, h = i - r * H;
                dagg[static_cast<size_t>(order[t0 + r]) * H + h] = dcur[i];
            }
            __syncthreads();
        }
        // da of this level is read by earlier levels of this same workgroup
        __threadfence_block();
        __syncthreads();
    }
}

// (d) inputs of the matrix-core chain kernel, in the bucket order of the direction whose chunks
// it walks (pd; the sweep being differentiated is sd = 1 - pd): the outside gradient of s_v and
// the ReLU gates of the node's layers, one byte per (node, column): bit 0 m_v > 0, bit 1 output
// of f's layer 0 > 0 (L = 2), bit 2 output of g's last layer > 0, bit 3 output of g's layer 0 > 0
// (L = 2).
struct GateSrc {
    const float *m;        // [n_tot, H] messages (output of f's last layer)
    const float *f0;       // output of f's layer 0 (L = 2)
    const float *g_last;   // output of g's last layer
    const float *g0;       // output of g's layer 0 (L = 2)
};

__global__ __launch_bounds__(kThreads) void k_bw_gates(GraphView gv, int H, int L, GateSrc src0, GateSrc src1,
                                                       uint8_t *__restrict__ mask4)
{
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= static_cast<size_t>(gv.n_tot) * H) return;
    for (int sd = 0; sd < 2; ++sd) {
        const GateSrc &gs = sd ? src1 : src0;
        int bits = fabsf(gs.m[idx]) > 0.0f ? 1 : 0;     // messages may carry a flag in their sign bit
        bits |= gs.g_last[idx] > 0.0f ? 4 : 0;
        if (L == 2) {
            bits |= gs.f0[idx] > 0.0f ? 2 : 0;
            bits |= gs.g0[idx] > 0.0f ? 8 : 0;
        }
        mask4[static_cast<size_t>(sd) * gv.n_tot * H + idx] = static_cast<uint8_t>(bits);
    }
}

// ------------------------------------------------------------------ 4. projection
// x_v = relu(W^T phi_v + b) feeds both directions: dx_v = (ds_td + ds_bu) masked by x_v > 0.
// Also writes phi_v, the input rows of the projection's weight gradient.
__global__ __launch_bounds__(kThreads) void k_bw_proj(GraphView gv, ModelView mv,
                                                      const float *__restrict__ feats,
                                                      const int32_t *__restrict__ placement,
                                                      const int32_t *__restrict__ cur_node,
                                                      const float *__restrict__ demb,
                                                      float *__restrict__ dx,
                                                      float *__restrict__ phi, int phi_ld)
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
    const bool is_cur = v - gv.node_off[b] == cur_node[b];
    if (is_cur) s += W[(2 + D) * H + h];
    s = fmaf(feats[v * 3 + 2], W[(3 + D) * H + h], s);
    const float g = demb[static_cast<size_t>(v) * 2 * H + h] + demb[static_cast<size_t>(v) * 2 * H + H + h];
    dx[idx] = s > 0.0f ? g : 0.0f;
    if (h < phi_ld) {                       // phi_ld >= F: columns past F are zero
        float p;
        if (h == 0) p = feats[v * 3 + 0];
        else if (h == 1) p = feats[v * 3 + 1];
        else if (h < 2 + D) p = (dev == h - 2) ? 1.0f : 0.0f;
        else if (h == 2 + D) p = is_cur ? 1.0f : 0.0f;
        else if (h == 3 + D) p = feats[v * 3 + 2];
        else p = 0.0f;
        phi[static_cast<size_t>(v) * phi_ld + h] = p;
    }
}

// The same with four columns per thread, for H a multiple of four (vector loads and stores; the
// per-node values are read once per four columns).  The sum takes its terms in the order of
// k_bw_proj, which is the forward pass's.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4p;
__global__ __launch_bounds__(kThreads) void k_bw_proj4(GraphView gv, ModelView mv,
                                                       const float *__restrict__ feats,
                                                       const int32_t *__restrict__ placement,
                                                       const int32_t *__restrict__ cur_node,
                                                       const float *__restrict__ demb,
                                                       float *__restrict__ dx,
                                                       float *__restrict__ phi, int phi_ld)
{
    const int H = mv.H, D = mv.D, q = H / 4;
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= static_cast<size_t>(gv.n_tot) * q) return;
    const int v = static_cast<int>(idx / q), h = 4 * static_cast<int>(idx - static_cast<size_t>(v) * q);
    const int b = gv.node_graph[v];
    const float *W = mv.blob + mv.proj.w;
    auto row = [&](int r) { return *reinterpret_cast<const f32x4p *>(W + static_cast<size_t>(r) * H + h); };
    const float f_time = feats[v * 3 + 0], f_size = feats[v * 3 + 1], f_vis = feats[v * 3 + 2];
    const int dev = placement[v];
    const bool on_dev = dev >= 0 && dev < D;
    const bool is_cur = v - gv.node_off[b] == cur_node[b];
    const f32x4p bias = *reinterpret_cast<const f32x4p *>(mv.blob + mv.proj.b + h);
    const f32x4p w0 = row(0), w1 = row(1), wd = row(2 + (on_dev ? dev : 0)), wc = row(2 + D), wv = row(3 + D);
    const float *de = demb + static_cast<size_t>(v) * 2 * H + h;
    const f32x4p g0 = *reinterpret_cast<const f32x4p *>(de), g1 = *reinterpret_cast<const f32x4p *>(de + H);
    f32x4p out;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        float s = bias[k];
        s = fmaf(f_time, w0[k], s);
        s = fmaf(f_size, w1[k], s);
        if (on_dev) s += wd[k];
        if (is_cur) s += wc[k];
        s = fmaf(f_vis, wv[k], s);
        out[k] = s > 0.0f ? g0[k] + g1[k] : 0.0f;
    }
    *reinterpret_cast<f32x4p *>(dx + static_cast<size_t>(v) * H + h) = out;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = h + k;
        if (c < phi_ld) {                   // phi_ld >= F: columns past F are zero
            float p;
            if (c == 0) p = f_time;
            else if (c == 1) p = f_size;
            else if (c < 2 + D) p = (dev == c - 2) ? 1.0f : 0.0f;
            else if (c == 2 + D) p = is_cur ? 1.0f : 0.0f;
            else if (c == 3 + D) p = f_vis;
            else p = 0.0f;
            phi[static_cast<size_t>(v) * phi_ld + c] = p;
        }
    }
}

// phi rows when H < F (more raw features than embedding columns): one thread per (node, feature).
__global__ __launch_bounds__(kThreads) void k_bw_phi(GraphView gv, ModelView mv,
                                                     const float *__restrict__ feats,
                                                     const int32_t *__restrict__ placement,
                                                     const int32_t *__restrict__ cur_node,
                                                     float *__restrict__ phi)
{
    const int D = mv.D, F = mv.F;
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= static_cast<size_t>(gv.n_tot) * F) return;
    const int v = static_cast<int>(idx / F), h = static_cast<int>(idx - static_cast<size_t>(v) * F);
    const int b = gv.node_graph[v];
    const int dev = placement[v];
    float p;
    if (h == 0) p = feats[v * 3 + 0];
    else if (h == 1) p = feats[v * 3 + 1];
    else if (h < 2 + D) p = (dev == h - 2) ? 1.0f : 0.0f;
    else if (h == 2 + D) p = (v - gv.node_off[b] == cur_node[b]) ? 1.0f : 0.0f;
    else p = feats[v * 3 + 2];
    phi[idx] = p;
}

// ------------------------------------------------------------------ dense layers on the matrix cores
// Y[row][j] = epi(bias[j] + sum_k X[row][k] Wt[j][k]) for a list of rows, H in {32, 64, 128} output
// columns (NJ tiles of 32) and K a multiple of 32.  A workgroup of four waves takes 128 rows; wave
// w multiplies rows 32 w .. 32 w + 31 by all columns; X and Wt go through LDS in chunks of 32 k.
// epi: optional ReLU, optional gate (Y = 0 where M[row][j] <= 0).  rows / n_rows_dev: optional row
// list and its length in device memory (the grid covers R rows; workgroups past the length exit).
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8w;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4v;

constexpr int kDenseKC = 32;                  // k per chunk
constexpr int kDenseRows = 128;               // rows per workgroup

// On the bf16 matrix cores at fp32 accuracy (operands split into three bf16 parts, six products
// kept: see k_wgrad_split).  The weights come in the transposed layout
// Wt[j][k] (row j holds the K inputs of output column j), so that both operands are contiguous
// along k: a 16-byte LDS cell holds the eight bf16 of one row (or output column) for eight
// consecutive k, and a fragment of v_mfma_f32_32x32x16_bf16 (lane = row, eight k) is one
// ds_read_b128.  A thread stages half cells: a float4 (coalesced along k: 128-byte row pieces),
// split in registers, three 8-byte stores; the row-group stride of 136 cells puts the two groups
// a store instruction touches on different halves of the banks.  One LDS buffer, the next chunk
// in registers meanwhile, two barriers per chunk; grid.z walks several row lists (z-th list,
// count, weights and bias: strides given) in one launch.
constexpr int kDsGS = 136;                    // cells between the row groups of the X parts
constexpr size_t dense_split_lds_bytes(int NJ) { return static_cast<size_t>(16) * 3 * 4 * (kDsGS + 32 * NJ + 8); }

template <int NJ>
__global__ __launch_bounds__(kThreads, 3) void k_dense_split(const float *__restrict__ X, int ldx,
                                                             const int32_t *__restrict__ rows,
                                                             const int32_t *__restrict__ n_rows_dev, int R, int K,
                                                             const float *__restrict__ Wt, int ldwt,
                                                             const float *__restrict__ bias, int relu,
                                                             const float *__restrict__ M, int ldm,
                                                             float *__restrict__ Y, int ldy, size_t list_stride,
                                                             size_t w_stride, size_t b_stride)
{
    constexpr int Hc = 32 * NJ, GSW = Hc + 8;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint2 *half_x = reinterpret_cast<uint2 *>(lds_raw);                 // [3][4][kDsGS] cells of two halves
    uint2 *half_w = half_x + 2 * 3 * 4 * kDsGS;                         // [3][4][GSW]
    const uint4 *cell_x = reinterpret_cast<const uint4 *>(half_x);
    const uint4 *cell_w = reinterpret_cast<const uint4 *>(half_w);
    rows += blockIdx.z * list_stride;
    if (n_rows_dev) R = min(R, n_rows_dev[blockIdx.z]);
    Wt += blockIdx.z * w_stride;
    if (bias) bias += blockIdx.z * b_stride;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lk = lane >> 5;
    const int tile0 = blockIdx.x * kDenseRows;
    if (tile0 >= R) return;                                // the whole workgroup, before any barrier

    // this thread's share of a chunk: float4 number (tid & 7) of the 32 k, of rows xr + 32 q and of
    // output columns xr + 32 q
    const int xr = tid >> 3, xc = (tid & 7) * 4;
    const int grp = xc >> 3, hf = (xc >> 2) & 1;
    const float *xsrc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int r = min(tile0 + xr + 32 * q, R - 1);
        xsrc[q] = X + static_cast<size_t>(rows ? rows[r] : r) * ldx + xc;
    }
    f32x4v xreg[4], wreg[NJ];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) xreg[q] = *reinterpret_cast<const f32x4v *>(xsrc[q] + k0);
#pragma unroll
        for (int q = 0; q < NJ; ++q)
            wreg[q] = *reinterpret_cast<const f32x4v *>(Wt + static_cast<size_t>(xr + 32 * q) * ldwt + k0 + xc);
    };
    auto put_half = [&](uint2 *cells, int stride, int c, const f32x4v &v) {
        auto top = [](float x) { return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u); };
        auto pack = [](float lo, float hi) {
            return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
        };
        float r[4], l[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            r[i] = v[i] - top(v[i]);
            l[i] = r[i] - top(r[i]);
        }
        cells[2 * ((0 * 4 + grp) * stride + c) + hf] = uint2{pack(v[0], v[1]), pack(v[2], v[3])};
        cells[2 * ((1 * 4 + grp) * stride + c) + hf] = uint2{pack(r[0], r[1]), pack(r[2], r[3])};
        cells[2 * ((2 * 4 + grp) * stride + c) + hf] = uint2{pack(l[0], l[1]), pack(l[2], l[3])};
    };
    auto stash = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) put_half(half_x, kDsGS, xr + 32 * q, xreg[q]);
#pragma unroll
        for (int q = 0; q < NJ; ++q) put_half(half_w, GSW, xr + 32 * q, wreg[q]);
    };

    f32x16 acc[NJ];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[jb][v] = 0.0f;

    const int n_chunks = K / kDenseKC;
    fetch(0);
    for (int c = 0; c < n_chunks; ++c) {
        stash();
        __syncthreads();
        if (c + 1 < n_chunks) fetch((c + 1) * kDenseKC);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int g = 2 * ks + lk;
            bf16x8w a[3];
#pragma unroll
            for (int p = 0; p < 3; ++p)
                a[p] = *reinterpret_cast<const bf16x8w *>(&cell_x[(p * 4 + g) * kDsGS + 32 * wave + li]);
            constexpr int JP = NJ > 1 ? 2 : 1;
            constexpr int pa[6] = {2, 0, 1, 1, 0, 0}, pb[6] = {0, 2, 1, 0, 1, 0};   // small products first
#pragma unroll
            for (int j0 = 0; j0 < NJ; j0 += JP) {
                bf16x8w b[JP][3];
#pragma unroll
                for (int u = 0; u < JP; ++u)
#pragma unroll
                    for (int p = 0; p < 3; ++p)
                        b[u][p] = *reinterpret_cast<const bf16x8w *>(&cell_w[(p * 4 + g) * GSW + 32 * (j0 + u) + li]);
#pragma unroll
                for (int t = 0; t < 6; ++t)
#pragma unroll
                    for (int u = 0; u < JP; ++u)
                        acc[j0 + u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pa[t]], b[u][pb[t]], acc[j0 + u], 0, 0, 0);
            }
        }
        __syncthreads();
    }

    float bj[NJ];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) bj[jb] = bias ? bias[32 * jb + li] : 0.0f;
    int orow[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int rc = min(tile0 + 32 * wave + 8 * (v / 4) + 4 * lk + (v % 4), R - 1);
        orow[v] = rows ? rows[rc] : rc;
    }
    auto finish = [&](auto gated) {
        // with gates: all gate values of a column tile are loaded before its first store (loads
        // and stores retire in order: a load behind a store would wait for it)
#pragma unroll
        for (int jb = 0; jb < NJ; ++jb) {
            float gate[16];
            if constexpr (decltype(gated)::value) {
#pragma unroll
                for (int v = 0; v < 16; ++v) gate[v] = M[static_cast<size_t>(orow[v]) * ldm + 32 * jb + li];
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int r = tile0 + 32 * wave + 8 * (v / 4) + 4 * lk + (v % 4);
                float y = acc[jb][v] + bj[jb];
                if (relu) y = fmaxf(y, 0.0f);
                if constexpr (decltype(gated)::value) y = gate[v] > 0.0f ? y : 0.0f;
                if (r < R) Y[static_cast<size_t>(orow[v]) * ldy + 32 * jb + li] = y;
            }
        }
    };
    if (M)
        finish(std::true_type{});
    else
        finish(std::false_type{});
}

// a_v = sum of the neighbours' messages, for every node and both directions (grid.y).
// Four columns per thread (H is a multiple of 32 on this path).
__global__ __launch_bounds__(kThreads) void k_bw_agg(GraphView gv, int H,
                                                     const float *__restrict__ msgs,
                                                     float *__restrict__ agg)
{
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int q = H / 4;
    if (idx >= static_cast<size_t>(gv.n_tot) * q) return;
    const int dir = blockIdx.y;
    const int v = static_cast<int>(idx / q), h = 4 * static_cast<int>(idx - static_cast<size_t>(v) * q);
    const float *msg = msgs + static_cast<size_t>(dir) * gv.n_tot * H;   // [2, n_tot, H] from the forward pass
    const int32_t *nbr_ptr = gv.nbr_ptr[dir], *nbr_idx = gv.nbr_idx[dir];
    f32x4v a{0.f, 0.f, 0.f, 0.f};
    for (int p = nbr_ptr[v]; p < nbr_ptr[v + 1]; ++p) {
        // messages are ReLU outputs; the matrix-core sweep keeps a flag in their sign bit
        const f32x4v m = *reinterpret_cast<const f32x4v *>(msg + static_cast<size_t>(nbr_idx[p]) * H + h);
        a += f32x4v{fabsf(m[0]), fabsf(m[1]), fabsf(m[2]), fabsf(m[3])};
    }
    *reinterpret_cast<f32x4v *>(agg + (static_cast<size_t>(dir) * gv.n_tot + v) * H + h) = a;
}

// Node set of every node and the three sets as row lists in ascending node order, in three
// steps with no atomics (the lists fix the summation order of l's weight gradients): per block
// of 256 nodes the number of nodes of each set; an exclusive scan over the blocks; the fill.
// The first step also copies the gradient of e_{v*} from dz.
__device__ __forceinline__ int node_class_of(const GraphView &gv, int v, const uint8_t *reach,
                                             const int32_t *cur_node, int single, int *graph)
{
    const int b = gv.node_graph[v];
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = cur_node[b];
    const int cur = (cl >= 0 && cl < n_b) ? n0 + cl : -1;
    *graph = b;
    return node_class_bw(v, cur, reach, gv.n_tot, single);
}

__global__ __launch_bounds__(kThreads) void k_bw_cls_count(GraphView gv, int H, int Z, int single,
                                                           const uint8_t *__restrict__ reach,
                                                           const int32_t *__restrict__ cur_node,
                                                           const float *__restrict__ dz,
                                                           uint8_t *__restrict__ cls,
                                                           int32_t *__restrict__ blk_cnt,
                                                           float *__restrict__ demb)
{
    __shared__ int wcnt[4][3];
    const int v = blockIdx.x * kThreads + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int k = -1, b = 0;
    if (v < gv.n_tot) {
        k = node_class_of(gv, v, reach, cur_node, single, &b);
        cls[v] = static_cast<uint8_t>(k);
    }
    for (int c = 1; c <= 3; ++c) {
        const unsigned long long m = __ballot(k == c);
        if (lane == 0) wcnt[wave][c - 1] = __popcll(m);
    }
    __syncthreads();
    if (threadIdx.x < 3)
        blk_cnt[blockIdx.x * 3 + threadIdx.x] = wcnt[0][threadIdx.x] + wcnt[1][threadIdx.x] +
                                                wcnt[2][threadIdx.x] + wcnt[3][threadIdx.x];
    if (k == 0)
        for (int i = 0; i < 2 * H; ++i) demb[static_cast<size_t>(v) * 2 * H + i] = dz[static_cast<size_t>(b) * Z + i];
}

// One workgroup: blk_cnt[blk][c] becomes the position of the block's first node of set c in
// list c; counts[c] = size of set c.
__global__ __launch_bounds__(kThreads) void k_bw_cls_scan(int n_blocks, int32_t *__restrict__ blk_cnt,
                                                          int32_t *__restrict__ counts)
{
    __shared__ int part[kThreads][3];
    const int tid = threadIdx.x;
    const int per = (n_blocks + kThreads - 1) / kThreads;
    const int lo = min(n_blocks, tid * per), hi = min(n_blocks, lo + per);
    int sum[3] = {0, 0, 0};
    for (int i = lo; i < hi; ++i)
        for (int c = 0; c < 3; ++c) sum[c] += blk_cnt[i * 3 + c];
    for (int c = 0; c < 3; ++c) part[tid][c] = sum[c];
    __syncthreads();
    if (tid < 3) {
        int run = 0;
        for (int t = 0; t < kThreads; ++t) {
            const int x = part[t][tid];
            part[t][tid] = run;
            run += x;
        }
        counts[tid] = run;
    }
    __syncthreads();
    int run[3] = {part[tid][0], part[tid][1], part[tid][2]};
    for (int i = lo; i < hi; ++i)
        for (int c = 0; c < 3; ++c) {
            const int x = blk_cnt[i * 3 + c];
            blk_cnt[i * 3 + c] = run[c];
            run[c] += x;
        }
}

__global__ __launch_bounds__(kThreads) void k_bw_cls_fill(GraphView gv, const uint8_t *__restrict__ cls,
                                                          const int32_t *__restrict__ blk_off,
                                                          int32_t *__restrict__ lists)
{
    __shared__ int wcnt[4][3];
    const int v = blockIdx.x * kThreads + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int k = v < gv.n_tot ? cls[v] : -1;
    int before = 0;
    for (int c = 1; c <= 3; ++c) {
        const unsigned long long m = __ballot(k == c);
        if (lane == 0) wcnt[wave][c - 1] = __popcll(m);
        if (k == c) before = __popcll(m & ((1ull << lane) - 1));
    }
    __syncthreads();
    if (k >= 1) {
        int pos = blk_off[blockIdx.x * 3 + k - 1] + before;
        for (int w = 0; w < wave; ++w) pos += wcnt[w][k - 1];
        lists[static_cast<size_t>(k - 1) * gv.n_tot + pos] = v;
    }
}

// Delta of l's last layer for every node: dP[set of the node][device of the node], gated by the
// layer's output; zero for a node whose device id is out of range (it was pooled nowhere).  Four
// columns per thread.
__global__ __launch_bounds__(kThreads) void k_bw_pool_seed(GraphView gv, int H, int G, int D,
                                                           const uint8_t *__restrict__ cls,
                                                           const int32_t *__restrict__ placement,
                                                           const float *__restrict__ dP,
                                                           const float *__restrict__ act,
                                                           float *__restrict__ dl)
{
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    const int q = H / 4;
    if (idx >= static_cast<size_t>(gv.n_tot) * q) return;
    const int v = static_cast<int>(idx / q), h = 4 * static_cast<int>(idx - static_cast<size_t>(v) * q);
    const int k = cls[v];
    if (k == 0) return;                       // the current node is in no set
    const int b = gv.node_graph[v];
    const int dev = placement[v];
    const bool ok = dev >= 0 && dev < D;
    const size_t at = static_cast<size_t>(v) * H + h;
    const f32x4v a = *reinterpret_cast<const f32x4v *>(act + at);
    f32x4v g{0.f, 0.f, 0.f, 0.f};
    if (ok) g = *reinterpret_cast<const f32x4v *>(dP + ((static_cast<size_t>(b) * 3 + (k - 1)) * G + (G == 1 ? 0 : dev)) * H + h);
    f32x4v o;
#pragma unroll
    for (int i = 0; i < 4; ++i) o[i] = a[i] > 0.0f ? g[i] : 0.0f;
    *reinterpret_cast<f32x4v *>(dl + at) = o;
}

// ------------------------------------------------------------------ 5. weight gradients
// partial[slab][i * J + j] = sum over the slab's rows r of A[r][i] * Dl[r][j]  (i in this
// workgroup's block of kWgI), partial[slab][I * J + j] = sum of Dl[r][j] (the bias).  Rows whose
// class byte differs from `want` are skipped when row_cls is given.  Thread (grp, j): column j,
// rows grp, grp + groups, ... of every staged batch; groups are added in order at the end.
__global__ __launch_bounds__(kThreads) void k_wgrad(const float *__restrict__ A, int lda,
                                                    const float *__restrict__ Dl, int ldd,
                                                    const uint8_t *__restrict__ row_cls, int want,
                                                    int R, int I, int J, int rows_per_slab,
                                                    float *__restrict__ partial)
{
    // (the matrix-core version below takes a row list instead of the class filter)
    __shared__ float a_s[kWgRB][kWgI];
    __shared__ int ok_s[kWgRB];
    __shared__ float red[kThreads * (kWgI + 1)];
    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kWgI, sl = blockIdx.y;
    const int r_beg = sl * rows_per_slab, r_end = min(R, r_beg + rows_per_slab);
    const int groups = kThreads / J;
    const int grp = tid / J, j = tid - grp * J;
    const bool active = grp < groups;
    float acc[kWgI];
#pragma unroll
    for (int ii = 0; ii < kWgI; ++ii) acc[ii] = 0.0f;
    float accb = 0.0f;
    for (int r0 = r_beg; r0 < r_end; r0 += kWgRB) {
        for (int idx = tid; idx < kWgRB * kWgI; idx += kThreads) {
            const int rr = idx / kWgI, ii = idx - rr * kWgI;
            const int row = r0 + rr;
            const bool ok = row < r_end && (!row_cls || row_cls[row] == want);
            a_s[rr][ii] = (ok && i0 + ii < I) ? A[static_cast<size_t>(row) * lda + i0 + ii] : 0.0f;
            if (ii == 0) ok_s[rr] = ok ? 1 : 0;
        }
        __syncthreads();
        if (active) {
            for (int rr = grp; rr < kWgRB; rr += groups) {
                if (!ok_s[rr]) continue;
                const float d = Dl[static_cast<size_t>(r0 + rr) * ldd + j];
#pragma unroll
                for (int ii = 0; ii < kWgI; ++ii) acc[ii] = fmaf(a_s[rr][ii], d, acc[ii]);
                accb += d;
            }
        }
        __syncthreads();
    }
    if (active) {
#pragma unroll
        for (int ii = 0; ii < kWgI; ++ii) red[(grp * (kWgI + 1) + ii) * J + j] = acc[ii];
        red[(grp * (kWgI + 1) + kWgI) * J + j] = accb;
    }
    __syncthreads();
    if (active && grp == 0) {
        float *dst = partial + static_cast<size_t>(sl) * (static_cast<size_t>(I) * J + J);
        for (int ii = 0; ii <= kWgI; ++ii) {
            float s = 0.0f;
            for (int gq = 0; gq < groups; ++gq) s += red[(gq * (kWgI + 1) + ii) * J + j];
            if (ii < kWgI) {
                if (i0 + ii < I) dst[static_cast<size_t>(i0 + ii) * J + j] = s;
            } else if (blockIdx.x == 0) {
                dst[static_cast<size_t>(I) * J + j] = s;
            }
        }
    }
}

// The same contraction on the matrix cores, for I a multiple of 32 and J in {32, 64, 128}:
// v_mfma_f32_32x32x2_f32 multiplies a 32 x 2 block of A^T by a 2 x 32 block of Dl in fp32, so two
// contraction rows are consumed per instruction (lanes 0-31 take the even row, lanes 32-63 the odd
// one; no split into bf16 parts).  A workgroup owns rows [128 blockIdx.x, +128) of the weight
// matrix (wave w: 32 of them) and all J columns, for one slab of contraction rows.  The rows of A
// and Dl go through LDS in chunks of 16, double buffered: every element is read from global
// memory once per workgroup (coalesced float4), the loads of chunk c + 1 travel during the 32
// matrix instructions of chunk c, and the ids of a row list are read one chunk further ahead.
// Row strides in LDS keep the two halves of a wave on different banks.
constexpr int kWgRC = 32;

constexpr int wgrad_ldd(int J) { return J == 128 ? 160 : 96; }
constexpr size_t wgrad_lds_bytes(int NJ) { return sizeof(float) * 2 * kWgRC * (160 + wgrad_ldd(32 * NJ)); }

template <int NJ>
__global__ __launch_bounds__(kThreads) void k_wgrad_mfma(const float *__restrict__ A, int lda,
                                                         const float *__restrict__ Dl, int ldd,
                                                         const int32_t *__restrict__ rows,
                                                         const int32_t *__restrict__ n_rows_dev,
                                                         int R, int I, int rows_per_slab,
                                                         float *__restrict__ partial)
{
    constexpr int J = 32 * NJ, LDA_S = 160, LDD_S = wgrad_ldd(J);
    constexpr int DT = kWgRC * J / 4;                      // float4 of a Dl chunk: 512, 256, 128
    constexpr int DQ = (DT + kThreads - 1) / kThreads;     // per thread: 2, 1, 1
    extern __shared__ float lds[];
    float *as = lds;                                       // [2][kWgRC][LDA_S]
    float *dsm = lds + 2 * kWgRC * LDA_S;                  // [2][kWgRC][LDD_S]
    if (n_rows_dev) R = min(R, *n_rows_dev);               // slabs past the list's end write zeros
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lk = lane >> 5;
    const int iw = blockIdx.x * 128, sl = blockIdx.y;
    const bool wave_on = iw + 32 * wave < I;
    const int r_beg = min(R, sl * rows_per_slab), r_end = min(R, r_beg + rows_per_slab);
    const int n_chunks = (r_end - r_beg + kWgRC - 1) / kWgRC;

    // this thread's pieces of a chunk: A rows ar + 8 q, floats ac .. ac + 3; Dl element 4 (tid + 256 q)
    const int ar = tid >> 5, ac = (tid & 31) * 4;
    const bool a_col_ok = iw + ac < I;
    constexpr int AQ = kWgRC / 8;                          // A pieces per thread and chunk
    int ida[AQ], idd[DQ];
    auto load_ids = [&](int r0) {
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int row = r0 + ar + 8 * q;
            ida[q] = row < r_end ? (rows ? rows[row] : row) : -1;
        }
#pragma unroll
        for (int q = 0; q < DQ; ++q) {
            const int e = (tid + kThreads * q) * 4;
            const int row = r0 + e / J;
            idd[q] = (e < kWgRC * J && row < r_end) ? (rows ? rows[row] : row) : -1;
        }
    };
    f32x4v areg[AQ], dreg[DQ];
    auto fetch = [&]() {
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const f32x4v v = *reinterpret_cast<const f32x4v *>(
                A + static_cast<size_t>(max(ida[q], 0)) * lda + (a_col_ok ? iw + ac : 0));
            areg[q] = (ida[q] >= 0 && a_col_ok) ? v : f32x4v{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int q = 0; q < DQ; ++q) {
            const int e = (tid + kThreads * q) * 4, c = e % J;
            const f32x4v v = *reinterpret_cast<const f32x4v *>(Dl + static_cast<size_t>(max(idd[q], 0)) * ldd + c);
            dreg[q] = idd[q] >= 0 ? v : f32x4v{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int q = 0; q < AQ; ++q)
            *reinterpret_cast<f32x4v *>(as + (buf * kWgRC + ar + 8 * q) * LDA_S + ac) = areg[q];
#pragma unroll
        for (int q = 0; q < DQ; ++q) {
            const int e = (tid + kThreads * q) * 4;
            if (e < kWgRC * J)
                *reinterpret_cast<f32x4v *>(dsm + (buf * kWgRC + e / J) * LDD_S + e % J) = dreg[q];
        }
    };

    f32x16 acc[NJ];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[jb][v] = 0.0f;
    float bsum[NJ];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) bsum[jb] = 0.0f;

    if (n_chunks > 0) {
        load_ids(r_beg);
        fetch();
        load_ids(r_beg + kWgRC);
        stash(0);
    }
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const int buf = c & 1;
        if (c + 1 < n_chunks) {
            fetch();                                       // chunk c + 1, ids read during chunk c - 1
            load_ids(r_beg + (c + 2) * kWgRC);
        }
        const float *ap = as + buf * kWgRC * LDA_S + lk * LDA_S + 32 * wave + li;
        const float *dp = dsm + buf * kWgRC * LDD_S + lk * LDD_S + li;
#pragma unroll
        for (int st = 0; st < kWgRC / 2; ++st) {
            const float a = ap[2 * st * LDA_S];
#pragma unroll
            for (int jb = 0; jb < NJ; ++jb) {
                const float b = dp[2 * st * LDD_S + 32 * jb];
                if (wave_on) acc[jb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[jb], 0, 0, 0);
                bsum[jb] += b;
            }
        }
        if (c + 1 < n_chunks) stash(buf ^ 1);
        __syncthreads();
    }
    if (!wave_on) return;
    float *dst = partial + static_cast<size_t>(sl) * (static_cast<size_t>(I) * J + J);
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = iw + 32 * wave + 8 * (v / 4) + 4 * lk + (v % 4);
            dst[static_cast<size_t>(i) * J + 32 * jb + li] = acc[jb][v];
        }
        const float other = __shfl_xor(bsum[jb], 32);
        if (blockIdx.x == 0 && wave == 0 && lk == 0) dst[static_cast<size_t>(I) * J + 32 * jb + li] = bsum[jb] + other;
    }
}

// The same contraction on the bf16 matrix cores at fp32 accuracy.  Every fp32 operand is split
// exactly into three bf16 parts by truncation (x = hi + mid + lo, 8 + 8 + 8 mantissa bits) and six
// of the nine products of parts are accumulated in fp32: hi hi, hi mid, mid hi, hi lo, lo hi,
// mid mid; the three left out are below 2^-24 of the product.  On v_mfma_f32_32x32x16_bf16 that
// is 2.7 times the rate of the fp32 instruction.
// A chunk is 32 contraction rows.  LDS holds the parts fragment-major: a 16-byte cell is the eight
// bf16 of one column for eight consecutive rows and the cells of consecutive columns are
// adjacent, so a fragment (lane = column, eight rows) is one conflict-free ds_read_b128.  A
// thread stages whole cells: eight rows of one column (the lanes of a wave on consecutive
// columns, 256-byte row segments), split in registers, three 16-byte stores.  The rows of chunk
// c + 1 are in flight in registers while chunk c is multiplied; the ids of a row list are staged
// in LDS one chunk further ahead.  Column sums of Dl (the bias gradient) are taken in fp32 from
// the staged values, by the thread that stages the column.

constexpr size_t wgrad_split_lds_bytes(int NJ)
{
    return static_cast<size_t>(16) * 3 * 4 * (128 + 32 * NJ) + sizeof(int32_t) * 2 * kWgRC + sizeof(float) * kThreads;
}

template <int NJ>
__global__ __launch_bounds__(kThreads, 3) void k_wgrad_split(const float *__restrict__ A, int lda,
                                                          const float *__restrict__ Dl, int ldd,
                                                          const int32_t *__restrict__ rows,
                                                          const int32_t *__restrict__ n_rows_dev,
                                                          int R, int I, int rows_per_slab,
                                                          float *__restrict__ partial, size_t list_stride,
                                                          size_t partial_stride)
{
    constexpr int J = 32 * NJ;
    constexpr int NDC = (4 * J + kThreads - 1) / kThreads;     // Dl cells per thread: 2, 1, 1
    // grid.z > 1: the same contraction over several row lists at once (list z, its length, its slabs)
    rows += blockIdx.z * list_stride;
    n_rows_dev += blockIdx.z;
    partial += blockIdx.z * partial_stride;
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint4 *cell_a = reinterpret_cast<uint4 *>(lds_raw);                       // [3 parts][4 row groups][128 columns]
    uint4 *cell_d = cell_a + 3 * 4 * 128;                                      // [3 parts][4 row groups][J columns]
    int32_t *tab = reinterpret_cast<int32_t *>(cell_d + 3 * 4 * J);           // [2][32] row ids of a chunk
    float *bsh = reinterpret_cast<float *>(tab + 2 * kWgRC);                  // [256] column sums at the end
    if (n_rows_dev) R = min(R, *n_rows_dev);               // slabs past the list's end write zeros
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 31, lk = lane >> 5;
    const int iw = blockIdx.x * 128, sl = blockIdx.y;
    const bool wave_on = iw + 32 * wave < I;
    const int r_beg = min(R, sl * rows_per_slab), r_end = min(R, r_beg + rows_per_slab);
    const int n_chunks = (r_end - r_beg + kWgRC - 1) / kWgRC;

    // this thread's cells: A column ca, row groups ga and ga + 2; Dl column cd, row groups of cell tid + 256 q
    const int ca = tid & 127, ga = tid >> 7;
    const bool a_col_ok = iw + ca < I;
    const int cd = tid % J;
    float av[2][8], dv[NDC][8];       // the values of the chunk in flight, unmasked
    uint32_t amask = 0, dmask = 0;    // bit 8 q + k: value [q][k] belongs to the slab
    // ids of rows 8 grp .. 8 grp + 7 of the chunk at r0: from the staged list, or the row numbers
    // themselves; -1 past the slab's end.  Straight-line code: the loads that follow are all
    // issued before the first of them is used.
    auto row_ids = [&](int r0, int slot, int grp, int (&ids)[8]) {
        const int4 t0 = *reinterpret_cast<const int4 *>(tab + slot * kWgRC + 8 * grp);
        const int4 t1 = *reinterpret_cast<const int4 *>(tab + slot * kWgRC + 8 * grp + 4);
        const int listed[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int r = r0 + 8 * grp + k;
            ids[k] = rows ? listed[k] : (r < r_end ? r : -1);
        }
    };
    auto fetch = [&](int r0, int slot) {
        int ida[2][8], idd[NDC][8];
#pragma unroll
        for (int q = 0; q < 2; ++q) row_ids(r0, slot, ga + 2 * q, ida[q]);
#pragma unroll
        for (int q = 0; q < NDC; ++q) {
            const int cell = tid + kThreads * q;
            row_ids(r0, slot, cell < 4 * J ? cell / J : 0, idd[q]);
        }
        const int col_a = a_col_ok ? iw + ca : 0;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k)    // (the launcher checks that 32-bit element offsets suffice)
                av[q][k] = A[static_cast<uint32_t>(max(ida[q][k], 0)) * static_cast<uint32_t>(lda) + static_cast<uint32_t>(col_a)];
#pragma unroll
        for (int q = 0; q < NDC; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k)
                dv[q][k] = Dl[static_cast<uint32_t>(max(idd[q][k], 0)) * static_cast<uint32_t>(ldd) + static_cast<uint32_t>(cd)];
        // which of them count: one bit per value
        amask = 0;
        dmask = 0;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k) amask |= (ida[q][k] >= 0 && a_col_ok) ? 1u << (8 * q + k) : 0u;
#pragma unroll
        for (int q = 0; q < NDC; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k)
                dmask |= (idd[q][k] >= 0 && tid + kThreads * q < 4 * J) ? 1u << (8 * q + k) : 0u;
    };
    // the three bf16 parts of eight values, eight to a 16-byte cell (masked: the values whose bit
    // of ok is clear count as zero)
    auto put_cells = [&](auto masked, uint4 *cells, int C, int grp, int c, const float (&v)[8], uint32_t ok) {
        uint32_t h[4], m[4], l[4];
        auto top = [](float x) { return __uint_as_float(__float_as_uint(x) & 0xFFFF0000u); };
        auto pack = [](float lo, float hi) {       // the upper halves of two floats in one word
            return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
        };
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float x0 = v[2 * k], x1 = v[2 * k + 1];
            if constexpr (decltype(masked)::value) {
                x0 = (ok >> (2 * k)) & 1u ? x0 : 0.0f;
                x1 = (ok >> (2 * k + 1)) & 1u ? x1 : 0.0f;
            }
            const float r0 = x0 - top(x0), r1 = x1 - top(x1);
            const float l0 = r0 - top(r0), l1 = r1 - top(r1);
            h[k] = pack(x0, x1);
            m[k] = pack(r0, r1);
            l[k] = pack(l0, l1);
        }
        cells[(0 * 4 + grp) * C + c] = uint4{h[0], h[1], h[2], h[3]};
        cells[(1 * 4 + grp) * C + c] = uint4{m[0], m[1], m[2], m[3]};
        cells[(2 * 4 + grp) * C + c] = uint4{l[0], l[1], l[2], l[3]};
    };
    float bsum = 0.0f;
    bool whole = false;               // the chunk in flight came in with fetch_whole(): nothing to mask
    auto stash = [&]() {
        if (whole) {
#pragma unroll
            for (int q = 0; q < 2; ++q) put_cells(std::false_type{}, cell_a, 128, ga + 2 * q, ca, av[q], 0u);
#pragma unroll
            for (int q = 0; q < NDC; ++q) {
                put_cells(std::false_type{}, cell_d, J, (tid + kThreads * q) / J, cd, dv[q], 0u);
#pragma unroll
                for (int k = 0; k < 8; ++k) bsum += dv[q][k];
            }
            return;
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) put_cells(std::true_type{}, cell_a, 128, ga + 2 * q, ca, av[q], amask >> (8 * q));
#pragma unroll
        for (int q = 0; q < NDC; ++q) {
            const int cell = tid + kThreads * q;
            if (cell < 4 * J) {
                put_cells(std::true_type{}, cell_d, J, cell / J, cd, dv[q], dmask >> (8 * q));
#pragma unroll
                for (int k = 0; k < 8; ++k) bsum += (dmask >> (8 * q + k)) & 1u ? dv[q][k] : 0.0f;
            }
        }
    };
    // A chunk that lies wholly inside the slab, for J >= 64: the row group of each of a thread's
    // cells is the same over its wave, so row ids and row addresses are scalars and a load costs no
    // vector arithmetic; nothing is masked (columns past I load column 0 and are zeroed here).
    auto fetch_whole = [&](auto listed, int r0, int slot) {
        constexpr bool kListed = decltype(listed)::value;
        // ids of the eight rows of a group, as scalars (all reads of the list first, then the loads)
        auto group_ids = [&](int grp, int (&ids)[8]) {
            if constexpr (kListed) {
                const int4 t0 = *reinterpret_cast<const int4 *>(tab + slot * kWgRC + 8 * grp);
                const int4 t1 = *reinterpret_cast<const int4 *>(tab + slot * kWgRC + 8 * grp + 4);
                const int v[8] = {t0.x, t0.y, t0.z, t0.w, t1.x, t1.y, t1.z, t1.w};
#pragma unroll
                for (int k = 0; k < 8; ++k) ids[k] = __builtin_amdgcn_readfirstlane(v[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 8; ++k) ids[k] = r0 + 8 * grp + k;
            }
        };
        int ida[2][8], idd[NDC][8];
#pragma unroll
        for (int q = 0; q < 2; ++q) group_ids(__builtin_amdgcn_readfirstlane(ga + 2 * q), ida[q]);
#pragma unroll
        for (int q = 0; q < NDC; ++q) group_ids(__builtin_amdgcn_readfirstlane((tid + kThreads * q) / J), idd[q]);
        const uint32_t col_a = a_col_ok ? iw + ca : 0;
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k) av[q][k] = (A + static_cast<size_t>(ida[q][k]) * lda)[col_a];
#pragma unroll
        for (int q = 0; q < NDC; ++q)
#pragma unroll
            for (int k = 0; k < 8; ++k) dv[q][k] = (Dl + static_cast<size_t>(idd[q][k]) * ldd)[static_cast<uint32_t>(cd)];
        if (!a_col_ok) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int k = 0; k < 8; ++k) av[q][k] = 0.0f;
        }
    };
    auto fetch_chunk = [&](int r0, int slot) {
        whole = J >= 64 && r0 + kWgRC <= r_end;
        if (!whole)
            fetch(r0, slot);
        else if (rows)
            fetch_whole(std::true_type{}, r0, slot);
        else
            fetch_whole(std::false_type{}, r0, slot);
    };
    auto list_id = [&](int r0) {                           // thread k < 32: id of row k of the chunk at r0
        return (rows && tid < kWgRC && r0 + tid < r_end) ? rows[r0 + tid] : -1;
    };

    f32x16 acc[NJ];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[jb][v] = 0.0f;

    if (tid < kWgRC) {
        tab[tid] = list_id(r_beg);
        tab[kWgRC + tid] = list_id(r_beg + kWgRC);
    }
    __syncthreads();
    if (n_chunks > 0) fetch_chunk(r_beg, 0);
    for (int c = 0; c < n_chunks; ++c) {
        const int next_id = list_id(r_beg + (c + 2) * kWgRC);      // in flight until the end of the iteration
        stash();                                                   // chunk c: registers -> cells
        __syncthreads();
        if (c + 1 < n_chunks) fetch_chunk(r_beg + (c + 1) * kWgRC, (c + 1) & 1);
        if (wave_on) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int grp = 2 * ks + lk;
                bf16x8w a[3];
#pragma unroll
                for (int p = 0; p < 3; ++p)
                    a[p] = *reinterpret_cast<const bf16x8w *>(&cell_a[(p * 4 + grp) * 128 + 32 * wave + li]);
                // two column tiles at a time, so that consecutive matrix instructions do not
                // wait for each other's accumulator
                constexpr int JP = NJ > 1 ? 2 : 1;
                constexpr int pa[6] = {2, 0, 1, 1, 0, 0}, pb[6] = {0, 2, 1, 0, 1, 0};   // small products first
#pragma unroll
                for (int j0 = 0; j0 < NJ; j0 += JP) {
                    bf16x8w b[JP][3];
#pragma unroll
                    for (int u = 0; u < JP; ++u)
#pragma unroll
                        for (int p = 0; p < 3; ++p)
                            b[u][p] = *reinterpret_cast<const bf16x8w *>(&cell_d[(p * 4 + grp) * J + 32 * (j0 + u) + li]);
#pragma unroll
                    for (int t = 0; t < 6; ++t)
#pragma unroll
                        for (int u = 0; u < JP; ++u)
                            acc[j0 + u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[pa[t]], b[u][pb[t]], acc[j0 + u], 0, 0, 0);
                }
            }
        }
        __syncthreads();
        if (tid < kWgRC) tab[(c & 1) * kWgRC + tid] = next_id;     // chunk c + 2; this half was last read for chunk c
    }
    // column sums of Dl: the threads that staged column j are tid = j, j + J, ...
    bsh[tid] = bsum;
    __syncthreads();
    float *dst = partial + static_cast<size_t>(sl) * (static_cast<size_t>(I) * J + J);
    if (blockIdx.x == 0 && tid < J) {
        float t = bsh[tid];
        for (int k = tid + J; k < kThreads && k < 4 * J; k += J) t += bsh[k];
        dst[static_cast<size_t>(I) * J + tid] = t;
    }
    if (!wave_on) return;
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = iw + 32 * wave + 8 * (v / 4) + 4 * lk + (v % 4);
            dst[static_cast<size_t>(i) * J + 32 * jb + li] = acc[jb][v];
        }
}

// out[idx] += sum over slabs.  A workgroup takes 32 consecutive entries; its eight thread rows
// each add the slabs q, q + 8, ... in order, and the eight sums are added in order: a fixed
// summation order with enough loads in flight.
// A slab holds src_count floats; entry idx of the output comes from entry idx of the slab, or from
// idx + src_skip for idx >= n_main (the bias row, when the slab's matrix was padded to more rows).
__global__ __launch_bounds__(kThreads) void k_wgrad_reduce(const float *__restrict__ partial, int n_slabs,
                                                           size_t count, size_t src_count, size_t n_main,
                                                           size_t src_skip, float *__restrict__ out)
{
    __shared__ float part[8][32];
    const int c = threadIdx.x & 31, q = threadIdx.x >> 5;
    const size_t idx = static_cast<size_t>(blockIdx.x) * 32 + c;
    const size_t src = idx < n_main ? idx : idx + src_skip;
    // four running sums per thread row (slabs q, q + 8, q + 16, q + 24, then again), added in order
    // at the end: still one fixed order, with four loads in flight
    float s4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (idx < count) {
        int sl = q;
        for (; sl + 24 < n_slabs; sl += 32) {
#pragma unroll
            for (int u = 0; u < 4; ++u) s4[u] += partial[static_cast<size_t>(sl + 8 * u) * src_count + src];
        }
#pragma unroll
        for (int u = 0; u < 3; ++u)     // at most three slabs are left
            if (sl + 8 * u < n_slabs) s4[u] += partial[static_cast<size_t>(sl + 8 * u) * src_count + src];
    }
    part[q][c] = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    __syncthreads();
    if (q == 0 && idx < count) {
        float t = part[0][c];
        for (int k = 1; k < 8; ++k) t += part[k][c];
        out[idx] += t;
    }
}

__global__ __launch_bounds__(kThreads) void k_fill_zero(float *__restrict__ p, size_t n)
{
    const size_t idx = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx < n) p[idx] = 0.0f;
}

int pick_rpt_bw(int H)
{
    int groups = kThreads / H;
    if (groups > kTile) groups = kTile;
    int rpt = 1;
    while (groups * rpt < kTile) rpt *= 2;
    return rpt;
}

template <typename K>
void allow_lds_bw(K kernel, size_t bytes)
{
    if (bytes > 48 * 1024)
        (void)hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
}

#define PL_DISPATCH_RPT(rpt, CALL) \
    switch (rpt) {                 \
        case 1: { CALL(1); break; }  \
        case 2: { CALL(2); break; }  \
        case 4: { CALL(4); break; }  \
        case 8: { CALL(8); break; }  \
        default: { CALL(16); break; } \
    }

// about two slabs per CU (768, one for each of the three workgroups a CU holds, was slower: the
// slab sums grow with the slab count)
int wgrad_rows_per_slab_cores(int64_t R)
{
    int64_t per = (R + 511) / 512;
    if (per < 64) per = 64;
    return static_cast<int>((per + 7) / 8 * 8);
}

int wgrad_rows_per_slab(int64_t R)
{
    int64_t per = (R + 383) / 384;
    if (per < 256) per = 256;
    return static_cast<int>((per + kWgRB - 1) / kWgRB * kWgRB);
}

}  // namespace

size_t wgrad_partial_floats(int64_t R, int I, int J)
{
    if (R <= 0) return 0;
    const int per_a = wgrad_rows_per_slab(R), per_b = wgrad_rows_per_slab_cores(R);
    const int64_t slabs = std::max((R + per_a - 1) / per_a, (R + per_b - 1) / per_b);
    return static_cast<size_t>(slabs) * (static_cast<size_t>(I) * J + J);
}

void launch_fill_zero(float *p, size_t n, hipStream_t s)
{
    if (n == 0) return;
    hipLaunchKernelGGL(k_fill_zero, dim3(static_cast<unsigned>((n + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       s, p, n);
}

// n_lists > 1 (matrix-core path with row lists only): the contraction is taken for n_lists row
// lists, list_stride apart with consecutive counts, in one launch, for the layers lys[0..n_lists).
void launch_wgrad(const float *A, int lda, const float *Dl, int ldd, const uint8_t *row_cls, int want,
                  const int32_t *list, const int32_t *list_count, int64_t R, const LayerRef &ly, float *partial,
                  float *grad, int generic, hipStream_t s, int I_pad = 0, int n_lists = 1, size_t list_stride = 0,
                  const LayerRef *lys = nullptr)
{
    // I_pad: A has I_pad >= n_in columns, the extra ones zero (lets a narrow layer use the matrix cores)
    if (R <= 0) return;
    const int I = I_pad ? I_pad : ly.n_in, J = ly.n_out;
    const bool cores = generic == 0 && I % 32 == 0 && (J == 32 || J == 64 || J == 128);
    const int per = cores ? wgrad_rows_per_slab_cores(R) : wgrad_rows_per_slab(R);
    const int slabs = static_cast<int>((R + per - 1) / per);
    if (cores) {
        // with a row list (the nodes of one set, ascending) the class filter is not needed
        const dim3 grid((I + 127) / 128, slabs, n_lists);
        const size_t slab_floats = static_cast<size_t>(slabs) * (static_cast<size_t>(I) * J + J);
        // the bf16-split kernel addresses its operands with 32-bit element offsets
        const bool small = static_cast<double>(R) * std::max(lda, ldd) < 4.0e9;   // the caller's duty if n_lists > 1
#define CALL(NJ)                                                                                                  \
    if (small) {                                                                                                  \
        allow_lds_bw(k_wgrad_split<NJ>, wgrad_split_lds_bytes(NJ));                                               \
        hipLaunchKernelGGL(k_wgrad_split<NJ>, grid, dim3(kThreads), wgrad_split_lds_bytes(NJ), s, A, lda, Dl, ldd, \
                           list, list_count, static_cast<int>(R), I, per, partial, list_stride, slab_floats);     \
    } else {                                                                                                      \
        allow_lds_bw(k_wgrad_mfma<NJ>, wgrad_lds_bytes(NJ));                                                      \
        hipLaunchKernelGGL(k_wgrad_mfma<NJ>, grid, dim3(kThreads), wgrad_lds_bytes(NJ), s, A, lda, Dl, ldd, list,  \
                           list_count, static_cast<int>(R), I, per, partial);                                     \
    }
        if (J == 32) { CALL(1); } else if (J == 64) { CALL(2); } else { CALL(4); }
#undef CALL
    } else {
        hipLaunchKernelGGL(k_wgrad, dim3((I + kWgI - 1) / kWgI, slabs), dim3(kThreads), 0, s, A, lda, Dl, ldd,
                           row_cls, want, static_cast<int>(R), I, J, per, partial);
    }
    const size_t n_main = static_cast<size_t>(ly.n_in) * J, count = n_main + J;
    const size_t src_count = static_cast<size_t>(I) * J + J;
    for (int z = 0; z < n_lists; ++z)
        hipLaunchKernelGGL(k_wgrad_reduce, dim3(static_cast<unsigned>((count + 31) / 32)), dim3(kThreads), 0, s,
                           partial + z * static_cast<size_t>(slabs) * src_count, slabs, count, src_count, n_main,
                           src_count - count, grad + (lys ? lys[z].w : ly.w));
}

namespace {

struct DenseCall {
    const float *X; int ldx;
    const int32_t *rows; const int32_t *n_rows_dev; int R; int K;
    const float *Wt; int ldwt;     // row j = the K inputs of output column j
    const float *bias; int relu;
    const float *M; int ldm;
    float *Y; int ldy;
    // n_lists row lists in one launch: z-th list at rows + z list_stride with count n_rows_dev[z],
    // weights at Wt + z w_stride, bias + z b_stride
    int n_lists = 1; size_t list_stride = 0, w_stride = 0, b_stride = 0;
};

void launch_dense(const DenseCall &c, int H, hipStream_t s)
{
    if (c.R <= 0) return;
    const dim3 grid((c.R + kDenseRows - 1) / kDenseRows, 1, c.n_lists);
#define CALL(NJ)                                                                                                 \
    allow_lds_bw(k_dense_split<NJ>, dense_split_lds_bytes(NJ));                                                  \
    hipLaunchKernelGGL(k_dense_split<NJ>, grid, dim3(kThreads), dense_split_lds_bytes(NJ), s, c.X, c.ldx, c.rows, \
                       c.n_rows_dev, c.R, c.K, c.Wt, c.ldwt, c.bias, c.relu, c.M, c.ldm, c.Y, c.ldy, c.list_stride, \
                       c.w_stride, c.b_stride)
    if (H == 32) { CALL(1); } else if (H == 64) { CALL(2); } else { CALL(4); }
#undef CALL
}

}  // namespace

void launch_backward(const GraphView &gv, const ModelView &mv, const float *blob_t, const Workspace &ws,
                     const GradWorkspace &gw, const ForwardArgs &fa, const BackwardArgs &ba, int k_sweeps,
                     int pool_chunks, int generic, const uint4 *wfrag_bw, const float *sweep_bias, int sweep_ws,
                     const float *keep, bool pool_kept, const StageMarks *marks, hipStream_t s)
{
    if (gv.B == 0) return;
    float *grad = ba.grad;
    const int H = mv.H, L = mv.L, G = mv.G, B = gv.B, n = gv.n_tot;
    const int rpt = pick_rpt_bw(H);
    const int n_slices = (mv.Z + 255) / 256;
    const size_t NH = static_cast<size_t>(n) * H;
    const size_t BG = static_cast<size_t>(B) * G;

    auto mark = [&](int stage, bool begin) {
        if (marks && marks->mark) marks->mark(marks->ctx, stage, begin, s);
    };
    // 1. head
    mark(PL_STAGE_BW_HEAD, true);
    hipLaunchKernelGGL(k_bw_head, dim3(B), dim3(kThreads), 0, s, gv, mv, blob_t, ws.hidp, n_slices, fa.cur_node,
                       ba.actions, ba.coeff, ba.entropy_coeff, ba.out_entropy, gw.hid, gw.dpre, gw.dlogit, gw.dz,
                       ba.out_logp);
    hipLaunchKernelGGL(k_bw_dz, dim3((mv.Z + kThreads - 1) / kThreads, (B + kDzGraphs - 1) / kDzGraphs), dim3(kThreads),
                       0, s, mv, B, blob_t, gw.dpre, gw.dz);
    {
        const size_t lds = sizeof(float) * 3 * kTile * H;
#define CALL(R)                                                                                          \
    allow_lds_bw(k_bw_head_sets<R>, lds);                                                                \
    hipLaunchKernelGGL(k_bw_head_sets<R>, dim3(3, B), dim3(kThreads), lds, s, gv, mv, blob_t, gw.pooled, \
                       gw.dz, gw.hin, gw.hact, gw.dh, gw.dP)
        // h_i works on the G rows of a set: as many rows per thread as that needs
        int groups = kThreads / H;
        if (groups > kTile) groups = kTile;
        if (groups < 1) groups = 1;
        int rpt_sets = 1;
        while (groups * rpt_sets < G) rpt_sets *= 2;
        PL_DISPATCH_RPT(rpt_sets, CALL)
#undef CALL
    }
    mark(PL_STAGE_BW_HEAD, false);
    mark(PL_STAGE_BW_POOL, true);
    // matrix-core dense layers: every output width of the embedding networks is H
    const bool dense = generic == 0 && (H == 32 || H == 64 || H == 128);
    // 2. pooling
    if (dense) {
        const int n_blocks = (n + kThreads - 1) / kThreads;
        hipLaunchKernelGGL(k_bw_cls_count, dim3(n_blocks), dim3(kThreads), 0, s, gv, H, mv.Z, mv.single_set, ws.reach,
                           fa.cur_node,
                           gw.dz, gw.cls, gw.blk_cnt, gw.demb);
        hipLaunchKernelGGL(k_bw_cls_scan, dim3(1), dim3(kThreads), 0, s, n_blocks, gw.blk_cnt, gw.counts);
        hipLaunchKernelGGL(k_bw_cls_fill, dim3(n_blocks), dim3(kThreads), 0, s, gv, gw.cls, gw.blk_cnt, gw.lists);
        for (int set = 0; set < 3; ++set) {
            const int32_t *list = gw.lists + static_cast<size_t>(set) * n, *cnt = gw.counts + set;
            const MlpRef &ln = mv.l[set];
            for (int l = 0; l < L && !pool_kept; ++l)     // kept: the forward pooling kernel wrote lact
                launch_dense({l == 0 ? ws.emb : gw.lact + static_cast<size_t>(l - 1) * NH, l == 0 ? 2 * H : H, list,
                              cnt, n, l == 0 ? 2 * H : H, blob_t + ln.layer[l].w, l == 0 ? 2 * H : H,
                              mv.blob + ln.layer[l].b, 1, nullptr, 0, gw.lact + static_cast<size_t>(l) * NH, H}, H, s);
        }
        // Where the forward pooling kernel kept l's layer outputs and its reverse is built, one pass
        // over the same tiles gives the deltas of l's layers and d e; else the dense-layer kernels.
        const bool stream_bw = pool_kept && ba.pool_bw_frag != nullptr;
        if (stream_bw) {
            launch_pool_stream_bw(gv, mv, ws, fa.placement, ba.pool_bw_frag, gw.lact, gw.dP, gw.cls, gw.dl, gw.demb, s);
        } else {
        hipLaunchKernelGGL(k_bw_pool_seed, dim3(static_cast<unsigned>((NH / 4 + kThreads - 1) / kThreads)),
                           dim3(kThreads), 0, s, gv, H, G, mv.D, gw.cls, fa.placement, gw.dP,
                           gw.lact + static_cast<size_t>(L - 1) * NH, gw.dl + static_cast<size_t>(L - 1) * NH);
        {
            // back through l's layers, the three sets' row lists in one launch each.  The weights go
            // in as they are stored (row i of a layer = the outputs fed by input i), which is the
            // transposed layout of this contraction; the three networks are equally far apart.
            const MlpRef &l0 = mv.l[0];
            const size_t w_stride = static_cast<size_t>(mv.l[1].layer[0].w - l0.layer[0].w);
            for (int l = L - 1; l >= 1; --l) {
                DenseCall c{gw.dl + static_cast<size_t>(l) * NH, H, gw.lists, gw.counts, n, H, mv.blob + l0.layer[l].w, H,
                            nullptr, 0, gw.lact + static_cast<size_t>(l - 1) * NH, H,
                            gw.dl + static_cast<size_t>(l - 1) * NH, H};
                c.n_lists = 3;
                c.list_stride = static_cast<size_t>(n);
                c.w_stride = w_stride;
                launch_dense(c, H, s);
            }
            for (int half = 0; half < 2; ++half) {   // the first layer is [2H, H]: inputs half H .. half H + H - 1
                DenseCall c{gw.dl, H, gw.lists, gw.counts, n, H,
                            mv.blob + l0.layer[0].w + static_cast<size_t>(half) * H * H, H, nullptr, 0, nullptr, 0,
                            gw.demb + half * H, 2 * H};
                c.n_lists = 3;
                c.list_stride = static_cast<size_t>(n);
                c.w_stride = w_stride;
                launch_dense(c, H, s);
            }
        }
        }
    } else {
        const size_t lds = sizeof(float) * kTile * 4 * H;
#define CALL(R)                                                                                             \
    allow_lds_bw(k_bw_pool<R>, lds);                                                                        \
    hipLaunchKernelGGL(k_bw_pool<R>, dim3(pool_chunks, B), dim3(kThreads), lds, s, gv, mv, blob_t, ws.emb,  \
                       ws.reach, fa.placement, fa.cur_node, gw.dP, gw.dz, gw.cls, gw.lact, gw.dl, gw.demb, \
                       pool_chunks)
        PL_DISPATCH_RPT(rpt, CALL)
#undef CALL
    }
    mark(PL_STAGE_BW_POOL, false);
    // 3. sweeps.  Where the layer outputs live: kept by the forward sweep (keep: slot 0 a_v, slots
    // 1 .. L g's layers, then f's layers but the last), or recomputed into fact / gact / agg.
    auto agg_of = [&](int dir) {
        return keep ? keep + dir * gw.dfg_stride : gw.agg + static_cast<size_t>(dir) * NH;
    };
    auto gact_of = [&](int dir, int l) {
        return keep ? keep + dir * gw.dfg_stride + static_cast<size_t>(1 + l) * NH
                    : gw.gact + (static_cast<size_t>(dir) * L + l) * NH;
    };
    auto fact_of = [&](int dir, int l) {       // l < L - 1 on the keep path (the last layer is ws.msg)
        return keep ? keep + dir * gw.dfg_stride + static_cast<size_t>(1 + L + l) * NH
                    : gw.fact + (static_cast<size_t>(dir) * L + l) * NH;
    };
    // one sweep at a time, from the last to the first: demb holds the outside gradient of the sweep's
    // output on entry and the gradient of its input on exit; the states and messages of an earlier
    // sweep come from the snapshots taken during the forward pass
    for (int j = k_sweeps - 1; j >= 0; --j) {
    const float *emb_j = j == k_sweeps - 1 ? ws.emb : ba.snap_emb + static_cast<size_t>(j) * 2 * NH;
    const float *msg_j = j == k_sweeps - 1 ? ws.msg : ba.snap_msg + static_cast<size_t>(j) * 2 * NH;
    mark(PL_STAGE_BW_ACTS, true);
    if (dense && !keep) {
        // the last layer of f is the message itself, which the forward pass left in msg_j (the
        // generic chain kernel reads it from fact, so there it is computed again)
        for (int dir = 0; dir < 2; ++dir)
            for (int l = 0; l + 1 < L || (l < L && !wfrag_bw); ++l) {
                const LayerRef &ly = mv.f[dir].layer[l];
                launch_dense({l == 0 ? emb_j + dir * H : gw.fact + (static_cast<size_t>(dir) * L + l - 1) * NH,
                              l == 0 ? 2 * H : H, nullptr, nullptr, n, H, blob_t + ly.w, H, mv.blob + ly.b, 1,
                              nullptr, 0, gw.fact + (static_cast<size_t>(dir) * L + l) * NH, H}, H, s);
            }
        hipLaunchKernelGGL(k_bw_agg, dim3(static_cast<unsigned>((NH / 4 + kThreads - 1) / kThreads), 2), dim3(kThreads),
                           0, s, gv, H, msg_j, gw.agg);
        for (int dir = 0; dir < 2; ++dir)
            for (int l = 0; l < L; ++l) {
                const LayerRef &ly = mv.g[dir].layer[l];
                launch_dense({l == 0 ? gw.agg + static_cast<size_t>(dir) * NH
                                     : gw.gact + (static_cast<size_t>(dir) * L + l - 1) * NH,
                              H, nullptr, nullptr, n, H, blob_t + ly.w, H, mv.blob + ly.b, 1, nullptr, 0,
                              gw.gact + (static_cast<size_t>(dir) * L + l) * NH, H}, H, s);
            }
    }
    {
        const size_t lds = sizeof(float) * 2 * kTile * H;
        const unsigned tiles = static_cast<unsigned>((n + kTile - 1) / kTile);
        if (!dense) {
#define CALL(R)                                                                                              \
    allow_lds_bw(k_bw_f_acts<R>, lds);                                                                       \
    allow_lds_bw(k_bw_g_acts<R>, lds);                                                                       \
    hipLaunchKernelGGL(k_bw_f_acts<R>, dim3(tiles, 2), dim3(kThreads), lds, s, gv, mv, emb_j, gw.fact);     \
    hipLaunchKernelGGL(k_bw_g_acts<R>, dim3(tiles, 2), dim3(kThreads), lds, s, gv, mv, gw.fact, gw.agg, gw.gact)
            PL_DISPATCH_RPT(rpt, CALL)
#undef CALL
        }
        if (wfrag_bw && !keep) {
            // the forward sweep that keeps activations also writes the gate bytes; otherwise they
            // are taken from the recomputed layer outputs here
            GateSrc src[2];
            for (int sd = 0; sd < 2; ++sd) {
                src[sd].m = dense ? msg_j + static_cast<size_t>(sd) * NH : fact_of(sd, L - 1);
                src[sd].f0 = L == 2 ? fact_of(sd, 0) : nullptr;
                src[sd].g_last = gact_of(sd, L - 1);
                src[sd].g0 = L == 2 ? gact_of(sd, 0) : nullptr;
            }
            hipLaunchKernelGGL(k_bw_gates, dim3(static_cast<unsigned>((NH + kThreads - 1) / kThreads)),
                               dim3(kThreads), 0, s, gv, H, L, src[0], src[1], gw.mask4);
        }
        mark(PL_STAGE_BW_ACTS, false);
        mark(PL_STAGE_BW_CHAIN, true);
        if (wfrag_bw) {
            launch_sweep_mfma_bw(gv, mv, wfrag_bw, sweep_bias, sweep_ws, fa.cur_node, gw.demb, gw.dagg, gw.mask4,
                                 gw.dfg, gw.dfg_stride, s);
        } else {
#define CALL(R)                                                                                            \
    allow_lds_bw(k_bw_sweep_generic<R>, lds);                                                              \
    hipLaunchKernelGGL(k_bw_sweep_generic<R>, dim3(B, 2), dim3(kThreads), lds, s, gv, mv, blob_t, gw.fact, \
                       gw.gact, gw.demb, gw.dagg, gw.dfg, gw.dfg_stride)
            PL_DISPATCH_RPT(rpt, CALL)
#undef CALL
        }
        mark(PL_STAGE_BW_CHAIN, false);
    }
    {
        mark(PL_STAGE_BW_WGRAD, true);
        for (int dir = 0; dir < 2; ++dir)
            for (int l = 0; l < L; ++l) {
                const float *dfl = gw.dfg + dir * gw.dfg_stride + static_cast<size_t>(l) * NH;
                const float *dgl = dfl + static_cast<size_t>(L) * NH;
                const float *fin = l == 0 ? emb_j + dir * H : fact_of(dir, l - 1);
                launch_wgrad(fin, l == 0 ? 2 * H : H, dfl, H, nullptr, 0, nullptr, nullptr, n, mv.f[dir].layer[l],
                             gw.partial, grad, generic, s);
                const float *gin = l == 0 ? agg_of(dir) : gact_of(dir, l - 1);
                launch_wgrad(gin, H, dgl, H, nullptr, 0, nullptr, nullptr, n, mv.g[dir].layer[l], gw.partial, grad, generic, s);
            }
        mark(PL_STAGE_BW_WGRAD, false);
    }
    }
    // 4. projection
    mark(PL_STAGE_BW_PROJ, true);
    {
        const size_t total = NH;
        if (H % 4 == 0)
            hipLaunchKernelGGL(k_bw_proj4, dim3(static_cast<unsigned>((total / 4 + kThreads - 1) / kThreads)),
                               dim3(kThreads), 0, s, gv, mv, fa.node_feats, fa.placement, fa.cur_node, gw.demb,
                               gw.dx, gw.phi, dense ? 32 : mv.F);
        else
            hipLaunchKernelGGL(k_bw_proj, dim3(static_cast<unsigned>((total + kThreads - 1) / kThreads)),
                               dim3(kThreads), 0, s, gv, mv, fa.node_feats, fa.placement, fa.cur_node, gw.demb,
                               gw.dx, gw.phi, dense ? 32 : mv.F);
        if (H < mv.F) {
            const size_t tf = static_cast<size_t>(n) * mv.F;
            hipLaunchKernelGGL(k_bw_phi, dim3(static_cast<unsigned>((tf + kThreads - 1) / kThreads)),
                               dim3(kThreads), 0, s, gv, mv, fa.node_feats, fa.placement, fa.cur_node, gw.phi);
        }
    }
    mark(PL_STAGE_BW_PROJ, false);
    // 5. weight gradients
    mark(PL_STAGE_BW_WGRAD, true);
    if (dense)   // raw features padded to 32 columns
        launch_wgrad(gw.phi, 32, gw.dx, H, nullptr, 0, nullptr, nullptr, n, mv.proj, gw.partial, grad, generic, s, 32);
    else
        launch_wgrad(gw.phi, mv.F, gw.dx, H, nullptr, 0, nullptr, nullptr, n, mv.proj, gw.partial, grad, generic, s);
    // the three sets' row lists in one launch per layer of l (all slabs of the three lists together
    // fill the chip; one list alone leaves most of its slabs empty)
    const bool sets_together = dense && static_cast<double>(n) * 2 * H < 4.0e9;
    if (sets_together)
        for (int l = 0; l < L; ++l) {
            const float *lin = l == 0 ? ws.emb : gw.lact + static_cast<size_t>(l - 1) * NH;
            const LayerRef lys[3] = {mv.l[0].layer[l], mv.l[1].layer[l], mv.l[2].layer[l]};
            launch_wgrad(lin, l == 0 ? 2 * H : H, gw.dl + static_cast<size_t>(l) * NH, H, gw.cls, 0, gw.lists,
                         gw.counts, n, lys[0], gw.partial, grad, generic, s, 0, 3, static_cast<size_t>(n), lys);
        }
    for (int set = 0; set < 3; ++set)
        for (int l = 0; l < L; ++l) {
            const float *lin = l == 0 ? ws.emb : gw.lact + static_cast<size_t>(l - 1) * NH;
            if (!sets_together)
                launch_wgrad(lin, l == 0 ? 2 * H : H, gw.dl + static_cast<size_t>(l) * NH, H, gw.cls, set + 1,
                             dense ? gw.lists + static_cast<size_t>(set) * n : nullptr,
                             dense ? gw.counts + set : nullptr, n, mv.l[set].layer[l], gw.partial, grad, generic, s);
            const float *hin = l == 0 ? gw.hin + static_cast<size_t>(set) * BG * H
                                      : gw.hact + (static_cast<size_t>(set) * L + l - 1) * BG * H;
            launch_wgrad(hin, H, gw.dh + (static_cast<size_t>(set) * L + l) * BG * H, H, nullptr, 0, nullptr, nullptr,
                         static_cast<int64_t>(BG), mv.h[set].layer[l], gw.partial, grad, generic, s);
        }
    launch_wgrad(ws.zbuf, mv.Z, gw.dpre, H, nullptr, 0, nullptr, nullptr, B, mv.pol1, gw.partial, grad, generic, s);
    launch_wgrad(gw.hid, H, gw.dlogit, mv.D, nullptr, 0, nullptr, nullptr, B, mv.pol2, gw.partial, grad, generic, s);
    mark(PL_STAGE_BW_WGRAD, false);
}

}  // namespace pl
