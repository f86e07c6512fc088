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

}  // namespace

void launch_episode_step(const GraphView &gv, int D, const float *logits, const float *uniforms,
                         const int32_t *order, int t, float *node_feats, int32_t *placement,
                         int32_t *cur_node, int32_t *out_action, float *out_logp, hipStream_t s)
{
    if (gv.B == 0) return;
    hipLaunchKernelGGL(k_episode_step, dim3((gv.B + 255) / 256), dim3(256), 0, s, gv, D, logits, uniforms, order,
                       t, node_feats, placement, cur_node, out_action, out_logp);
}

}  // namespace pl
