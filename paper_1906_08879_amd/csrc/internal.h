// Internal declarations shared by the host layout builder, the C ABI and the kernels.
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <string>
#include <vector>

#include "placeto.h"
#include "sweep_plan.h"

namespace pl {

constexpr int kMaxD = 16;
constexpr int kMaxH = 256;
constexpr int kMaxLayers = 4;
constexpr int kMaxSweeps = 8;

void set_error(const std::string &msg);
int fail(int code, const std::string &msg);
int hip_fail(hipError_t e, const char *what);

#define PL_HIP(call)                                             \
    do {                                                         \
        hipError_t e__ = (call);                                 \
        if (e__ != hipSuccess) return ::pl::hip_fail(e__, #call); \
    } while (0)

// ---- host-side layout of a batch (Section 2.2 step 2 needs parents and children of every
// node and an order in which all of a node's neighbours are final before the node).
struct HostLayout {
    int32_t B = 0;
    int64_t n_tot = 0, e_tot = 0;
    int32_t max_depth = 0;
    std::vector<int64_t> node_off;   // [B+1]
    std::vector<int64_t> edge_off;   // [B+1]
    std::vector<int64_t> par_ptr;    // [n_tot+1] into par_idx
    std::vector<int64_t> chi_ptr;    // [n_tot+1]
    std::vector<int32_t> par_idx;    // [e_tot] graph-local ids, ascending per node
    std::vector<int32_t> chi_idx;    // [e_tot]
    std::vector<int32_t> td_level;   // [n_tot]
    std::vector<int32_t> bu_level;   // [n_tot]
    std::vector<int32_t> td_order;   // [n_tot] graph-local ids by (level, id)
    std::vector<int32_t> bu_order;   // [n_tot]
    std::vector<int32_t> depth;      // [B] number of levels (same in both directions)
    std::vector<int64_t> lvl_off;    // [B+1] offset of graph b's level pointers
    std::vector<int32_t> td_lvl_ptr; // [lvl_off[B]] per graph depth+1 positions into its order
    std::vector<int32_t> bu_lvl_ptr; // same for bottom-up
    // graphs of the same topology (the rollouts of one graph) share what depends on the
    // topology alone: graph b uses the plan of template tmpl[b]; tmpl_graph[t] is a graph with it
    int32_t n_templates = 0;
    std::vector<int32_t> tmpl;       // [B]
    std::vector<int32_t> tmpl_graph; // [n_templates]
};

int build_layout(int32_t B, const int32_t *n_nodes, const int32_t *n_edges,
                 const int32_t *edge_src, const int32_t *edge_dst, HostLayout *out);
// The layout of R copies of the one graph of `one`, equal to what build_layout gives for the
// graph repeated R times, with all copies sharing one template.
int replicate_layout(const HostLayout &one, int32_t R, HostLayout *out);

// ---- device-side view of a batch, passed to kernels by value
struct GraphView {
    int32_t B;
    int32_t n_tot;
    const int32_t *node_off;   // [B+1]
    const int32_t *lvl_off;    // [B+1]
    // index 0 = top-down (neighbours = parents), 1 = bottom-up (neighbours = children)
    const int32_t *nbr_ptr[2]; // [n_tot+1]
    const int32_t *nbr_idx[2]; // [e_tot] GLOBAL node ids
    const int32_t *order[2];   // [n_tot] GLOBAL node ids by (graph, level, id)
    const int32_t *lvl_ptr[2]; // per graph depth+1 GLOBAL positions into order
    const int32_t *node_graph; // [n_tot] graph of each node
    const int32_t *pos[2];     // [n_tot] bucket position of each node (inverse of order)
    const int32_t *tmpl;       // [B] which plan (distinct topology) graph b uses
    SweepPlanView plan[2];     // per direction
};

// ---- parameters: offsets (in floats) of every layer inside the fp32 device blob
struct LayerRef {
    int32_t w;      // offset of the [in,out] matrix
    int32_t b;      // offset of the bias
    int32_t n_in;
    int32_t n_out;
};

struct MlpRef {
    LayerRef layer[kMaxLayers];
};

struct ModelView {
    int32_t D, H, L, G, Z, F;
    int32_t single_set;      // 1: every node other than v* belongs to the first node set
    const float *blob;       // fp32 (bf16-rounded values when the model stores bf16)
    LayerRef proj;
    MlpRef f[2], g[2];       // [direction]
    MlpRef l[3], h[3];       // [set]: parents, children, parallel
    LayerRef pol1, pol2;
};

// ---- the policy network's hidden unit j and logit d of graph b (Appendix A.7), in float64 from
// the partial products of its first layer; one definition for the forward and the reverse pass.
__device__ __forceinline__ double policy_hidden(const ModelView &mv, const double *__restrict__ hidp,
                                                int n_slices, int B, int b, int j)
{
    double s = static_cast<double>(mv.blob[mv.pol1.b + j]);
    for (int sl = 0; sl < n_slices; ++sl) s += hidp[(static_cast<size_t>(sl) * B + b) * mv.H + j];
    return s > 0.0 ? s : 0.0;
}

__device__ __forceinline__ float policy_logit(const ModelView &mv, const double *hid, int d)
{
    const float *W = mv.blob + mv.pol2.w;
    double s = static_cast<double>(mv.blob[mv.pol2.b + d]);
    for (int k = 0; k < mv.H; ++k) s = fma(hid[k], static_cast<double>(W[k * mv.D + d]), s);
    return static_cast<float>(s);
}

// ---- scratch owned by a batch for one (D, H)
struct Workspace {
    unsigned char *base = nullptr;  // the one allocation that holds every buffer but reach (null: not owned)
    float *emb = nullptr;       // [n_tot, 2H]  [td ; bu]
    float *msg = nullptr;       // [2, n_tot, H]
    float *xb = nullptr;        // [2, n_tot, H]  sweep input in bucket order (matrix-core path)
    float4 *featb = nullptr;    // [n_tot] raw-feature records in node order (matrix-core path)
    uint8_t *reach = nullptr;   // [2, n_tot]   0: descendant-of-v* bit, 1: ancestor-of-v* bit
    float *partial = nullptr;   // [B, n_chunks_max, 3G, H] pooling partial sums
    float *zbuf = nullptr;      // [B, Z] policy inputs
    double *hidp = nullptr;     // [ceil(Z / 256), B, H] partial products of policy layer 1 (float64 sums)
    int32_t *klist = nullptr;   // [n_tot] node ids grouped by (set, device group), per graph (matrix-core pooling)
    int32_t *koff = nullptr;    // [B][3 kMaxD + 1] first position of every key within its graph
    int32_t n_chunks = 0;
    int32_t H = 0, G = 0;
};

// ---- kernel launchers (kernels_generic.hip)
struct ForwardArgs {
    const float *node_feats;
    const int32_t *placement;
    const int32_t *cur_node;
    float *out_logits;
    float *out_probs;
    float *out_pooled;
};

constexpr int kPoolChunk = 128;   // nodes per pooling workgroup

void launch_project(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                    const ForwardArgs &fa, bool to_emb, bool to_xb, hipStream_t s);
void launch_sweep_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                          const ForwardArgs &fa, bool write_reach, hipStream_t s);
void launch_reach_only(const GraphView &gv, const int32_t *cur_node, uint8_t *reach, int n_max, int e_max,
                       int depth_max, hipStream_t s);
void launch_classes(const GraphView &gv, const int32_t *cur_node, const uint8_t *reach,
                    uint8_t *out_class, hipStream_t s);
void launch_pool_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                         const ForwardArgs &fa, hipStream_t s);
void launch_head_generic(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                         const ForwardArgs &fa, int max_chunks, hipStream_t s);

// ---- MDP transition (kernels_episode.hip)
void launch_episode_step(const GraphView &gv, int D, const float *logits, const float *uniforms,
                         const int32_t *order, int t, float *node_feats, int32_t *placement,
                         int32_t *cur_node, int32_t *out_action, float *out_logp, hipStream_t s);

void launch_episode_apply(const GraphView &gv, int D, const int32_t *actions, const int32_t *order, int t,
                          float *node_feats, int32_t *placement, int32_t *cur_node, hipStream_t s);
void launch_reinforce_coeff(int T, int B, int n_groups, const float *rewards, const int32_t *group,
                            float *coeff, float *baseline, hipStream_t s);

// ---- run-time simulator of a placement (kernels_simulator.hip); n_max / e_max: largest graph
size_t simulator_lds_bytes(int n_max, int e_max);
int launch_simulate(const GraphView &gv, int D, int n_max, int e_max, const float *node_feats,
                    const int32_t *placement, float inv_bw, bool per_child, float *out_runtime,
                    int32_t *out_events, hipStream_t s);

int launch_simulate_reward(const GraphView &gv, int D, int n_max, int e_max, const float *node_feats,
                           const int32_t *placement, float inv_bw, bool per_child, float mem_limit, float penalty,
                           float *op_start, float *op_end, float *arrival, float *arrival_last, float *alloc,
                           float *free_t, float *runtime, float *out_peak, float *out_reward, int32_t *out_events,
                           hipStream_t s);

// ---- matrix-core pooling (kernels_pool_mfma.hip); writes ws.partial as [B, kPoolSlices, 3G, H]
constexpr int kPoolSlices = 4;
bool pool_mfma_supported(int H, int L, int weight_dtype);
void pack_pool_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                       std::vector<float> *bias);
// fragments of the streaming pooling kernel (weights as A operands); bf16 weights at H = 128
bool pool_stream_supported(int H, int L, int weight_dtype);
void pack_pool_stream_weights(const ModelView &mv, const float *blob, std::vector<uint16_t> *frag);
// the reverse of the streaming pooling kernel (two-layer l): deltas of l's layers and d e of every
// pooled node from the kept layer outputs; reads the sort (ws.klist, ws.koff) of the forward pass
bool pool_stream_bw_supported(int H, int L, int weight_dtype);
void pack_pool_stream_bw_weights(const ModelView &mv, const float *blob, std::vector<uint16_t> *frag);
void launch_pool_stream_bw(const GraphView &gv, const ModelView &mv, const Workspace &ws, const int32_t *placement,
                           const uint4 *frag, const float *lact, const float *dP, const uint8_t *cls, float *dl,
                           float *demb, hipStream_t s);
// returns the number of slices per graph that ws.partial holds afterwards
int launch_pool_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                     const ForwardArgs &fa, const uint4 *wfrag, const uint4 *afrag, const float *bias, int WS,
                     float *keep, hipStream_t s);

// ---- policy gradient (kernels_backward.hip): buffers owned by a batch for one (D, H, L)
struct GradWorkspace {
    float *fact = nullptr, *gact = nullptr;   // [2, L, n_tot, H] layer outputs of f and g
    float *agg = nullptr, *dagg = nullptr;    // [2, n_tot, H] gathered sums and their gradients
    float *dfg = nullptr;                     // per direction [2L, n_tot, H] layer deltas of f, then of g,
                                              // then H spare floats; dfg_stride floats per direction
    size_t dfg_stride = 0;
    float *keep = nullptr;                    // per direction [2L, n_tot, H]: a_v and layer outputs stored by
                                              // the forward sweep (same stride as dfg)
    float *snap_emb = nullptr, *snap_msg = nullptr;   // k >= 2 sweeps: states and messages after every
                                              // sweep but the last, [k - 1][2 n_tot H] each
    int32_t snap_sweeps = 0;
    uint8_t *mask4 = nullptr;                 // [2 n_tot + 1, H] ReLU gates per (sweep direction, node, column)
    float *lact = nullptr, *dl = nullptr;     // [L, n_tot, H] layer outputs / deltas of l (own set)
    float *demb = nullptr;                    // [n_tot, 2H] gradient of the embeddings
    float *dx = nullptr;                      // [n_tot, H] delta of the projection
    float *phi = nullptr;                     // [n_tot, F] raw feature rows
    uint8_t *cls = nullptr;                   // [n_tot] node set of every node
    int32_t *counts = nullptr;                // [4] sizes of the three node sets
    int32_t *blk_cnt = nullptr;               // [ceil(n_tot / 256), 3] per-block counts, then offsets
    int32_t *lists = nullptr;                 // [3, n_tot] nodes of each set
    float *pooled = nullptr, *dP = nullptr;   // [B, 3, G, H]
    float *hin = nullptr;                     // [3, B G, H] inputs of h per set
    float *hact = nullptr, *dh = nullptr;     // [3, L, B G, H]
    float *dz = nullptr;                      // [B, Z]
    float *hid = nullptr, *dpre = nullptr;    // [B, H] policy hidden layer and its delta
    float *dlogit = nullptr;                  // [B, D]
    float *partial = nullptr;                 // slab sums of the weight-gradient contraction
    int32_t H = 0, G = 0, L = 0, D = 0;
};

// Optional per-stage timing hook: called at the beginning and the end of every stage of a pass.
struct StageMarks {
    void *ctx;
    void (*mark)(void *ctx, int stage, bool begin, hipStream_t s);
};

size_t wgrad_partial_floats(int64_t R, int I, int J);
void launch_fill_zero(float *p, size_t n, hipStream_t s);
// what a reverse pass is asked for (device arrays; the last three may be null)
struct BackwardArgs {
    const int32_t *actions;
    const float *coeff;
    const float *entropy_coeff;
    float *grad;
    float *out_logp;
    float *out_entropy;
    // states [k - 1][n_tot, 2H] and messages [k - 1][2, n_tot, H] after every sweep but the last
    const float *snap_emb;
    const float *snap_msg;
    // fragments of the reverse streaming pooling kernel, or null (then the dense-layer kernels do it)
    const uint4 *pool_bw_frag = nullptr;
};

void launch_backward(const GraphView &gv, const ModelView &mv, const float *blob_t, const Workspace &ws,
                     const GradWorkspace &gw, const ForwardArgs &fa, const BackwardArgs &ba, int k_sweeps,
                     int pool_chunks, int generic, const uint4 *wfrag_bw, const float *sweep_bias, int sweep_ws,
                     const float *keep, bool pool_kept, const StageMarks *marks, hipStream_t s);

// ---- matrix-core sweep (kernels_mfma.hip)
bool sweep_mfma_supported(int H, int L, int weight_dtype);
void pack_sweep_weights(const ModelView &mv, const float *blob, int WS, std::vector<uint16_t> *frag,
                        std::vector<float> *bias, bool reverse = false);
void launch_sweep_mfma_bw(const GraphView &gv, const ModelView &mv, const uint4 *wfrag, const float *bias,
                          int WS, const int32_t *cur_node, float *demb, float *dagg, uint8_t *mask4,
                          float *delta, size_t delta_stride, hipStream_t s);
void launch_sweep_mfma(const GraphView &gv, const ModelView &mv, const Workspace &ws,
                       const ForwardArgs &fa, const uint4 *wfrag, const float *bias, int WS,
                       bool first_sweep, bool more_sweeps, float *keep, size_t keep_stride, uint8_t *gates,
                       hipStream_t s);

}  // namespace pl
