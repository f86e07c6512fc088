// One MDP transition (Section 2.1) for every graph of a batch, on the device: the sampled
// action updates the current node's placement, the node is marked visited, and the next node
// of the visiting order becomes current.  One thread per graph: the work is B x D numbers.
#include "internal.h"

namespace pl {

namespace {

__global__ __launch_bounds__(256) void k_episode_step(GraphView gv, int D, const float *__restrict__ logits,
                                                      const float *__restrict__ uniforms,
                                                      const int32_t *__restrict__ order, int t,
                                                      float *__restrict__ node_feats,
                                                      int32_t *__restrict__ placement,
                                                      int32_t *__restrict__ cur_node,
                                                      int32_t *__restrict__ out_action,
                                                      float *__restrict__ out_logp)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= gv.B) return;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = cur_node[b];
    if (cl < 0 || cl >= n_b) {             // the graph's episode is over (or the state is invalid)
        cur_node[b] = -1;
        if (out_action) out_action[b] = -1;
        if (out_logp) out_logp[b] = 0.0f;
        return;
    }
    // softmax over the D logits (Appendix A.7) and inverse CDF over devices 0 .. D-1:
    // the first device whose cumulative weight exceeds u x total
    float e[kMaxD];
    float m = -INFINITY;
    for (int d = 0; d < D; ++d) m = fmaxf(m, logits[static_cast<size_t>(b) * D + d]);
    float total = 0.0f;
    for (int d = 0; d < D; ++d) {
        e[d] = expf(logits[static_cast<size_t>(b) * D + d] - m);
        total += e[d];
    }
    const float thr = uniforms[b] * total;
    int a = D - 1;
    float c = 0.0f;
    for (int d = 0; d < D; ++d) {
        c += e[d];
        if (c > thr) {
            a = d;
            break;
        }
    }
    if (out_action) out_action[b] = a;
    if (out_logp) out_logp[b] = logits[static_cast<size_t>(b) * D + a] - m - logf(total);
    placement[n0 + cl] = a;
    node_feats[static_cast<size_t>(n0 + cl) * 3 + 2] = 1.0f;
    cur_node[b] = (t + 1 < n_b) ? order[n0 + t + 1] : -1;
}

// The same transition with a given action (replay of a recorded episode): nothing is sampled.
// A graph whose episode is over, or whose action is outside [0, D), only has its current node
// set to -1.
__global__ __launch_bounds__(256) void k_episode_apply(GraphView gv, int D, const int32_t *__restrict__ actions,
                                                       const int32_t *__restrict__ order, int t,
                                                       float *__restrict__ node_feats,
                                                       int32_t *__restrict__ placement,
                                                       int32_t *__restrict__ cur_node)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= gv.B) return;
    const int n0 = gv.node_off[b], n_b = gv.node_off[b + 1] - n0;
    const int cl = cur_node[b];
    const int a = actions[b];
    if (cl < 0 || cl >= n_b || a < 0 || a >= D) {
        cur_node[b] = -1;
        return;
    }
    placement[n0 + cl] = a;
    node_feats[static_cast<size_t>(n0 + cl) * 3 + 2] = 1.0f;
    cur_node[b] = (t + 1 < n_b) ? order[n0 + t + 1] : -1;
}

// Weights of the REINFORCE sum (appendix "REINFORCE Algorithm", Eq. 1): the return that follows
// every decision, G[t][b] = sum_{t' >= t} r[t'][b] (one thread per rollout, from the last step
// backwards), the per-step baseline of every group of rollouts (mean of G[t][.] over the group,
// members added in ascending order), and their difference.
__global__ __launch_bounds__(256) void k_returns(int T, int B, const float *__restrict__ rewards,
                                                 float *__restrict__ coeff)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    float g = 0.0f;
    for (int t = T - 1; t >= 0; --t) {
        g += rewards[static_cast<size_t>(t) * B + b];
        coeff[static_cast<size_t>(t) * B + b] = g;
    }
}

__global__ __launch_bounds__(256) void k_baseline(int T, int B, int n_groups, const float *__restrict__ G,
                                                  const int32_t *__restrict__ group,
                                                  float *__restrict__ baseline)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= T * n_groups) return;
    const int t = idx / n_groups, g = idx - t * n_groups;
    float sum = 0.0f;
    int cnt = 0;
    for (int b = 0; b < B; ++b)
        if (group[b] == g) {
            sum += G[static_cast<size_t>(t) * B + b];
            ++cnt;
        }
    baseline[idx] = cnt ? sum / static_cast<float>(cnt) : 0.0f;
}

__global__ __launch_bounds__(256) void k_advantage(int T, int B, int n_groups, const int32_t *__restrict__ group,
                                                   const float *__restrict__ baseline,
                                                   float *__restrict__ coeff)
{
    const int idx = blockIdx.x * 256 + threadIdx.x;
    if (idx >= T * B) return;
    const int t = idx / B, b = idx - t * B;
    const int g = group[b];
    if (g >= 0 && g < n_groups) coeff[idx] -= baseline[static_cast<size_t>(t) * n_groups + g];
}

}  // namespace

void launch_episode_apply(const GraphView &gv, int D, const int32_t *actions, const int32_t *order, int t,
                          float *node_feats, int32_t *placement, int32_t *cur_node, hipStream_t s)
{
    if (gv.B == 0) return;
    hipLaunchKernelGGL(k_episode_apply, dim3((gv.B + 255) / 256), dim3(256), 0, s, gv, D, actions, order, t,
                       node_feats, placement, cur_node);
}

void launch_reinforce_coeff(int T, int B, int n_groups, const float *rewards, const int32_t *group,
                            float *coeff, float *baseline, hipStream_t s)
{
    if (T <= 0 || B <= 0) return;
    hipLaunchKernelGGL(k_returns, dim3((B + 255) / 256), dim3(256), 0, s, T, B, rewards, coeff);
    if (n_groups <= 0) return;
    hipLaunchKernelGGL(k_baseline, dim3((T * n_groups + 255) / 256), dim3(256), 0, s, T, B, n_groups, coeff, group,
                       baseline);
    hipLaunchKernelGGL(k_advantage, dim3((T * B + 255) / 256), dim3(256), 0, s, T, B, n_groups, group, baseline,
                       coeff);
}

void launch_episode_step(const GraphView &gv, int D, const float *logits, const float *uniforms,
                         const int32_t *order, int t, float *node_feats, int32_t *placement,
                         int32_t *cur_node, int32_t *out_action, float *out_logp, hipStream_t s)
{
    if (gv.B == 0) return;
    hipLaunchKernelGGL(k_episode_step, dim3((gv.B + 255) / 256), dim3(256), 0, s, gv, D, logits, uniforms, order,
                       t, node_feats, placement, cur_node, out_action, out_logp);
}

}  // namespace pl
