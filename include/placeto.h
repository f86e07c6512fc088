/*
 * placeto.h — C ABI of the MI355X (gfx950) library for Placeto's policy forward pass.
 *
 * The library evaluates, for a batch of independent computation graphs, the placement
 * policy of "Placeto: Learning Generalizable Device Placement Algorithms for Distributed
 * Machine Learning" (Section 2.2 and Appendix A.7): raw per-node features, two-way
 * message passing over the DAG, pooling over the current node's parent / child / parallel
 * sets, and a two-layer policy network with a softmax over devices.  Every step runs in
 * HIP kernels; there is no CPU fallback.
 *
 * General rules
 *   - Every function returns PL_OK (0) or a negative pl_status; no exception crosses the
 *     boundary.  pl_last_error() gives a thread-local message for the last failure.
 *   - "host" pointers are ordinary process memory; "dev" pointers are HIP device memory on
 *     the current device.  The library never frees or keeps caller memory.
 *   - Handles are created and destroyed by the library and are bound to the device that
 *     was current when they were first used by a device call.
 *   - A forward call is asynchronous on the given stream.  Two calls that use the same
 *     pl_graph_batch must not overlap in time: the batch owns the intermediate buffers.
 *   - Device-resident state is not range-checked by default (out-of-range values are contained,
 *     see pl_embed_forward).  With PL_VALIDATE=1 in the environment, pl_embed_forward(_ex),
 *     pl_policy_gradient(_ex), pl_episode_run and pl_episode_gradient first synchronise the stream,
 *     copy placement, cur_node (and actions) to the host and return PL_ERR_RANGE, launching
 *     nothing, if a device id or action is outside [0, D) or a current node outside its graph
 *     (in the two episode calls a cur_node of -1, a finished graph, is accepted).
 */
#ifndef PLACETO_H
#define PLACETO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PL_OK = 0,
    PL_ERR_NULL = -1,       /* a required pointer is NULL                               */
    PL_ERR_SHAPE = -2,      /* a size or configuration value is out of the supported range */
    PL_ERR_RANGE = -3,      /* a node id, device id or edge endpoint is out of range    */
    PL_ERR_SELF_LOOP = -4,  /* an edge (v, v)                                           */
    PL_ERR_DUP_EDGE = -5,   /* the same (src, dst) pair twice in one graph              */
    PL_ERR_CYCLE = -6,      /* the graph is not acyclic                                 */
    PL_ERR_HIP = -7,        /* a HIP runtime call failed (message has the HIP error)    */
    PL_ERR_NOMEM = -8,      /* host allocation failed                                   */
    PL_ERR_STATE = -9       /* a handle is not in the state the call needs              */
} pl_status;

/* Network configuration.  Appendix A.7: the message-passing and aggregation networks are
 * feed-forward with ReLU; the policy head has two layers and a softmax output. */
typedef struct {
    int32_t D;               /* number of devices, 1..16                                 */
    int32_t H;               /* embedding width, 1..256                                  */
    int32_t n_layers;        /* layers in each of f, g, l_i, h_i; 1..4 (the paper uses 1) */
    int32_t k_sweeps;        /* repetitions of the message passing (Section 2.2 step 2), 0..8 */
    int32_t group_by_device; /* 1: pool per (set, device); 0: per set only, as printed   */
    int32_t weight_dtype;    /* PL_WEIGHTS_FP32 or PL_WEIGHTS_BF16                       */
    int32_t single_set;      /* 0: the three node sets of Section 2.2 step 3; 1: every node
                                other than v* is pooled in the first set (the "simple aggregator"
                                of the paper's comparison of policy architectures; with
                                k_sweeps = 0 on top of it nothing of the graph structure is used;
                                k_sweeps = 0 alone is its "simple partitioner")          */
} pl_model_cfg;

enum { PL_WEIGHTS_FP32 = 0, PL_WEIGHTS_BF16 = 1 };

typedef struct pl_graph_batch pl_graph_batch;  /* opaque: CSR, levels, buckets, buffers */
typedef struct pl_weights pl_weights;          /* opaque: device copy of the parameters */

/* ---- graphs (Section 2: a DAG G(V,E) of op groups; an op receives tensors from its
 * parents).  All arguments are host memory.
 *   B          number of graphs (0 is allowed and gives an empty batch)
 *   n_nodes    [B]  nodes per graph, each >= 1
 *   n_edges    [B]  edges per graph, each >= 0
 *   edge_src, edge_dst  [sum n_edges]  concatenated in batch order, graph-local node ids;
 *              dst consumes src's output, so src is a PARENT of dst.  Edge order is free.
 * The grouped graph of the paper is a simple DAG: self loops, repeated edges and cycles
 * are refused (PL_ERR_SELF_LOOP / PL_ERR_DUP_EDGE / PL_ERR_CYCLE), endpoints outside
 * [0, n_nodes[b]) give PL_ERR_RANGE.  Builds, on the host: parent and child CSR (neighbour
 * lists ascending by id), longest-path levels from the roots (td) and from the leaves
 * (bu), and level buckets ordered by (level, node id).  Device copies are made on first
 * use by a device call.  *out is owned by the library until pl_graph_batch_destroy. */
int pl_graph_batch_create(int32_t B, const int32_t *n_nodes, const int32_t *n_edges,
                          const int32_t *edge_src, const int32_t *edge_dst,
                          pl_graph_batch **out);
/* A batch of R copies of ONE graph: the batch of independent rollouts of the same graph over
 * which the appendix's REINFORCE section averages its per-step baseline.  The result behaves in
 * every call exactly like pl_graph_batch_create on the graph repeated R times (same layout, same
 * results bit for bit); the host builds the layout once instead of R times, and what depends on
 * the topology alone (the message-passing kernel's gather plan) exists once on the device and is
 * read by all R copies.  Arguments as above for one graph; R >= 1. */
int pl_graph_batch_create_replicated(int32_t n_nodes, int32_t n_edges, const int32_t *edge_src,
                                     const int32_t *edge_dst, int32_t R, pl_graph_batch **out);
int pl_graph_batch_destroy(pl_graph_batch *g);   /* NULL is accepted */

/* Sizes of a batch: any output pointer may be NULL.  max_depth = largest number of levels
 * of any graph in the batch. */
int pl_graph_batch_info(const pl_graph_batch *g, int32_t *B, int64_t *n_tot, int64_t *e_tot,
                        int32_t *max_depth);

/* Levels of every node, host arrays [N_tot] in batch order.  td_level(v) = 0 for a node
 * without parents, else 1 + max over parents; bu_level symmetric over children. */
int pl_graph_batch_levels(const pl_graph_batch *g, int32_t *td_level, int32_t *bu_level);

/* The host-side layout, for inspection and tests.  Any pointer may be NULL.
 *   par_ptr, chi_ptr   [N_tot + 1]  offsets into par_idx / chi_idx (batch-wide)
 *   par_idx, chi_idx   [E_tot]      graph-local neighbour ids, ascending within a node
 *   td_order, bu_order [N_tot]      graph-local node ids of each graph, sorted by
 *                                   (level, id); graph b occupies its node range */
int pl_graph_batch_layout(const pl_graph_batch *g, int64_t *par_ptr, int32_t *par_idx,
                          int64_t *chi_ptr, int32_t *chi_idx, int32_t *td_order,
                          int32_t *bu_order);

/* Section 2.2 step 3: the sets of the current node v* of every graph.
 *   cur_node   dev [B]      graph-local id of v*
 *   out_class  dev [N_tot]  0 = v*, 1 = S_parents (can reach v*), 2 = S_children
 *                           (reachable from v*), 3 = S_parallel (neither)
 * Asynchronous on `stream` (a hipStream_t, NULL = default stream). */
int pl_node_classes(pl_graph_batch *g, const int32_t *cur_node, uint8_t *out_class,
                    void *stream);
/* The same call under its debugging name. */
int pl_debug_node_classes(pl_graph_batch *g, const int32_t *cur_node, uint8_t *out_class,
                          void *stream);

/* ---- parameters.  The blob holds, for every layer, a row-major [in, out] matrix followed
 * by `out` biases, in this order: input projection (D+4 -> H); f top-down, g top-down,
 * f bottom-up, g bottom-up (n_layers x H -> H each); l for the parent, child, parallel
 * sets (2H -> H, then H -> H); h for the same three (H -> H); policy layer 1
 * ((2 + 3G) H -> H, G = D or 1) and policy layer 2 (H -> D).
 * With PL_WEIGHTS_BF16 every matrix is rounded to bfloat16 (nearest even) on upload and
 * biases stay fp32; accumulation is fp32 in either case. */
size_t pl_weights_count(const pl_model_cfg *cfg);       /* 0 if cfg is invalid */
int pl_weights_create(const pl_model_cfg *cfg, const float *host_blob, size_t n_floats,
                      pl_weights **out);
int pl_weights_destroy(pl_weights *w);                  /* NULL is accepted */

/* Kernel selection for forward passes that use `w`: 0 (default) = the fastest kernels that
 * cover the configuration (matrix-core sweeps for H in {32, 64, 128} with bf16 weights,
 * H in {32, 64} with fp32 weights, n_layers <= 2); 1 = the generic fp32 kernels, which
 * cover every supported configuration.  Both compute the same function. */
int pl_weights_set_path(pl_weights *w, int32_t path);

/* ---- the forward pass (Section 2.2 steps 1-3 + policy head, Appendix A.7).
 *   node_feats  dev [N_tot, 3] fp32  per node: run time, output size, is-visited flag
 *                                    (Section 2.1 features 1, 2 and 4)
 *   placement   dev [N_tot] int32    current device of every node, in [0, D) (feature 3)
 *   cur_node    dev [B] int32        graph-local id of the node being placed (feature 5)
 *   out_logits  dev [B, D] fp32      pre-softmax policy outputs
 * The one-hot device and the is-current flag are derived inside the library.  A device id
 * outside [0, D) contributes an all-zero one-hot and is pooled nowhere; a cur_node outside
 * its graph gives NaN logits for that graph; neither writes out of bounds.
 * The first call on a batch for a given (D, H) allocates the batch's intermediate buffers
 * (and is therefore not capturable into a HIP graph); later calls only launch kernels. */
int pl_embed_forward(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                     const int32_t *cur_node, const pl_weights *w, float *out_logits,
                     void *stream);

/* Same, with optional extra outputs (NULL to skip):
 *   out_probs     dev [B, D]        softmax of the logits
 *   out_node_emb  dev [N_tot, 2H]   [top-down ; bottom-up] embedding of every node
 *   out_pooled    dev [B, 3, G, H]  summed l_i outputs per (set, device group)
 *   out_class     dev [N_tot] uint8 the node sets of Section 2.2 step 3 exactly as this pass's
 *                                   pooling used them (coded as in pl_node_classes): taken from
 *                                   the reachability bits that the message-passing kernels of this
 *                                   very call left behind, not from a separate traversal */
int pl_embed_forward_ex(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                        const int32_t *cur_node, const pl_weights *w, float *out_logits,
                        float *out_probs, float *out_node_emb, float *out_pooled,
                        uint8_t *out_class, void *stream);

/* ---- for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid it): pl_embed_forward with its intermediate buffers
 * (embeddings, messages, bucketed features, reachability bytes, pooling partial sums, policy
 * inputs) in a fixed block of device memory that is part of the library image, 32 MiB per
 * device (pl_embed_forward_static_limit), instead of buffers allocated on the batch's first call.
 * It calls no hipMalloc / hipFree and creates no events; it only launches kernels on `stream`.
 *   - The batch must be on the device already: pl_graph_batch_upload(g) makes the device copies
 *     of the index data (it allocates; call it once at set-up, with the device current that the
 *     later calls run on), else PL_ERR_STATE.  pl_weights handles are on the device from creation.
 *   - pl_embed_forward_static_bytes(g, w) is the size the call needs, about
 *     N_tot (24 H + 22) bytes; beyond the limit the call returns PL_ERR_SHAPE and launches nothing.
 *   - Every call on a device uses that device's one block, which keeps the last call's contents
 *     (what must read as zero is cleared by a small kernel at the start of each call): calls
 *     that overlap in time on one device race, whatever batches they use; calls on one stream,
 *     or otherwise ordered, are safe.  Stage timing (pl_profile_enable) does not cover it.
 * Arguments and results as pl_embed_forward; out_probs [B, D] may be NULL. */
int pl_graph_batch_upload(pl_graph_batch *g);
size_t pl_embed_forward_static_limit(void);
size_t pl_embed_forward_static_bytes(const pl_graph_batch *g, const pl_weights *w);
int pl_embed_forward_static(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                            const int32_t *cur_node, const pl_weights *w, float *out_logits,
                            float *out_probs, void *stream);

/* ---- the MDP transition (Section 2.1) on the device, for every graph of the batch: an
 * action a is drawn from softmax(logits[b]) (Appendix A.7) by inverse CDF, i.e. the first
 * device d whose cumulative probability exceeds uniforms[b]; the current node takes device a,
 * is marked visited, and node order[t + 1] of the graph becomes the current node (-1 after
 * the graph's last node, at which point the graph's episode is over).
 *   logits      dev [B, D] fp32     output of the forward pass on the state before the step
 *   uniforms    dev [B] fp32        numbers in [0, 1), drawn by the caller
 *   order       dev [N_tot] int32   per graph a permutation of its graph-local node ids,
 *                                   concatenated: the visiting order of the episode
 *   t                               index of this step in the episode (cur_node[b] is order[t])
 *   node_feats  dev [N_tot, 3]      in/out: the visited flag (column 2) of the current node := 1
 *   placement   dev [N_tot] int32   in/out: the current node's device := a
 *   cur_node    dev [B] int32       in/out: := order[t + 1] or -1
 *   out_action  dev [B] int32       a, or -1 for a graph whose episode is over (NULL to skip)
 *   out_logp    dev [B] fp32        log softmax(logits[b])[a], 0 for such a graph (NULL to skip)
 * A graph whose cur_node is outside the graph is left unchanged (cur_node := -1).
 * Asynchronous on `stream`; allocates nothing once the batch is on the device. */
int pl_episode_step(pl_graph_batch *g, int32_t D, const float *logits, const float *uniforms,
                    const int32_t *order, int32_t t, float *node_feats, int32_t *placement,
                    int32_t *cur_node, int32_t *out_action, float *out_logp, void *stream);

/* n_steps times { forward pass, transition }, steps t0 .. t0 + n_steps - 1 of the episode,
 * all enqueued on `stream` without any host synchronisation (Section 2.1: an episode is |V|
 * such steps).  Arguments as above, and
 *   uniforms     dev [n_steps, B]
 *   logits       dev [B, D], or [n_steps, B, D] when keep_logits != 0 (every step's logits)
 *   out_actions  dev [n_steps, B] or NULL;  out_logp  dev [n_steps, B] or NULL */
int pl_episode_run(pl_graph_batch *g, const pl_weights *w, float *node_feats, int32_t *placement,
                   int32_t *cur_node, const int32_t *order, const float *uniforms, int32_t t0,
                   int32_t n_steps, float *logits, int32_t keep_logits, int32_t *out_actions,
                   float *out_logp, void *stream);

/* ---- the policy gradient of one batch of decisions (appendix "REINFORCE Algorithm", Eq. 1:
 * theta <- theta + eta * sum_i grad_theta log pi_theta(a_i | s_i) * (sum_{i' >= i} r_i' - b_i)).
 * For the B states given as in pl_embed_forward, with the action taken in each and one scalar
 * per state (the caller's return-minus-baseline), computes
 *     grad (+)= sum_b coeff[b] * d/d theta log softmax(logits_theta(s_b))[actions[b]]
 * by a forward pass followed by a reverse pass through the policy head, the pooling, the two
 * message-passing directions (levels in reverse order) and the input projection.
 *   actions     dev [B] int32   device chosen for the current node, in [0, D)
 *   coeff       dev [B] fp32    scalar multiplying the state's gradient
 *   accumulate                  0: grad is overwritten; else the sum is added to it (the sum
 *                               over the steps of an episode is built by successive calls)
 *   grad        dev [pl_weights_count] fp32, laid out like the parameter blob (with
 *                               PL_WEIGHTS_BF16 the derivative is taken at the rounded weights)
 *   out_logits  dev [B, D] fp32 logits of the forward pass (required)
 *   out_logp    dev [B] fp32    log pi(a_b | s_b); NULL to skip
 * A graph whose cur_node or action is out of range adds nothing and gets out_logp = NaN.
 * ReLU's derivative at 0 is taken as 0.  With k_sweeps >= 2 the states and messages after every
 * sweep but the last are copied aside during the forward pass ((k_sweeps - 1) x 4 N_tot H floats
 * more) and the sweeps are differentiated from the last to the first.  The
 * first call on a batch allocates the buffers of the reverse pass (about (14 n_layers + 10)
 * x N_tot x H floats); later calls only launch kernels.  Asynchronous on `stream`; summation
 * orders are fixed, so equal inputs give bit-equal gradients. */
int pl_policy_gradient(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                       const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                       const float *coeff, int32_t accumulate, float *grad, float *out_logits,
                       float *out_logp, void *stream);

/* Same, with the entropy term that Appendix A.7 ("Entropy") adds to the loss to encourage
 * exploration: grad (+)= sum_b [ coeff[b] * d log pi(a_b | s_b) + entropy_coeff[b] * d H(pi(. | s_b)) ]
 * / d theta, H(pi) = - sum_d pi_d log pi_d (its derivative with respect to logit d is
 * - pi_d (log pi_d + H)).
 *   entropy_coeff  dev [B] fp32  the entropy factor of every state, or NULL for none
 *   out_entropy    dev [B] fp32  H(pi(. | s_b)), NaN for a graph whose cur_node is out of range; NULL to skip
 * A graph whose cur_node or action is out of range adds nothing for either term. */
int pl_policy_gradient_ex(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                          const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                          const float *coeff, const float *entropy_coeff, int32_t accumulate, float *grad,
                          float *out_logits, float *out_logp, float *out_entropy, void *stream);

/* The weights of that sum for T steps of B rollouts (Eq. 1: the return after each decision minus
 * a baseline; the baseline of step i is the average of that return over the independent
 * rollouts of the same graph):
 *     G[t][b] = sum_{t' >= t} rewards[t'][b]
 *     out_baseline[t][g] = mean of G[t][b] over the rollouts b with group[b] == g (0 if none)
 *     out_coeff[t][b] = G[t][b] - out_baseline[t][group[b]]
 *   rewards       dev [T, B] fp32   reward after step t of rollout b (0 after a rollout's end)
 *   group         dev [B] int32     id in [0, n_groups) shared by the rollouts of one graph; an id
 *                                   outside that range keeps the plain return
 *   out_coeff     dev [T, B] fp32;  out_baseline  dev [T, n_groups] fp32
 * n_groups = 0 gives the plain returns (group and out_baseline may then be NULL).  fp32 sums in a
 * fixed order (steps from the last backwards, rollouts ascending).  Asynchronous on `stream`;
 * allocates nothing. */
int pl_reinforce_coeff(int32_t T, int32_t B, const float *rewards, const int32_t *group, int32_t n_groups,
                       float *out_coeff, float *out_baseline, void *stream);

/* The whole sum of Eq. 1 for steps t0 .. t0 + n_steps - 1 of a recorded episode: for every step,
 * pl_policy_gradient on the current state with that step's actions and weights (accumulating
 * into grad), then the transition of Section 2.1 with the recorded action (as pl_episode_step,
 * nothing sampled), all enqueued on `stream` without host synchronisation.
 *   node_feats, placement, cur_node   dev, in/out: the state at step t0 (e.g. a copy of the
 *                                     state the rollout started from); advanced by n_steps
 *   order         dev [N_tot]         the visiting order used by the rollout
 *   actions       dev [n_steps, B]    e.g. out_actions of pl_episode_run
 *   coeff         dev [n_steps, B]    e.g. out_coeff of pl_reinforce_coeff
 *   entropy_coeff dev [n_steps, B]    entropy factors as in pl_policy_gradient_ex, or NULL
 *   accumulate                        0: grad is overwritten by the sum; else added to
 *   grad          dev [pl_weights_count];  logits  dev [B, D] scratch (last step's logits)
 *   out_logp      dev [n_steps, B] or NULL: log pi(a | s) of every replayed decision (NaN once a
 *                                     graph's episode is over)
 * Same behaviour as pl_policy_gradient_ex otherwise. */
int pl_episode_gradient(pl_graph_batch *g, const pl_weights *w, float *node_feats, int32_t *placement,
                        int32_t *cur_node, const int32_t *order, const int32_t *actions, const float *coeff,
                        const float *entropy_coeff, int32_t t0, int32_t n_steps, int32_t accumulate, float *grad,
                        float *logits, float *out_logp, void *stream);

/* ---- run time of a placement from the event-driven simulator of the paper's appendix
 * ("Simulator"), for every graph of the batch: per device a FIFO queue of runnable operations
 * and a FIFO queue of outgoing tensors, one operation per device and one transfer per bus at a
 * time, transfers overlapping compute; the result is the timestamp of the last op-done event.
 * This is the run time r of the reward R(p); pl_simulate_reward adds the peak-memory term.
 *   node_feats     dev [N_tot, 3]  column 0: run time of the operation, column 1: size of its output
 *   placement      dev [N_tot]     device of every node, in [0, D)
 *   inv_bandwidth                  seconds per unit of output size (a transfer takes size x this)
 *   out_runtime    dev [B] fp32    simulated run time; NaN for a graph with a device id outside [0, D)
 *   out_events     dev [B] int32   events processed (operations + transfers), -1 for such a graph; NULL to skip
 * Ties are broken as follows: roots are queued in ascending node id, children are visited in
 * ascending node id, an output crosses once per destination device, events are ordered by
 * (float32 timestamp, creation number), idle devices are started before idle buses, both in
 * ascending index.  A graph must fit in LDS: fewer than 65535 nodes and edges and
 * 18 n + 13 e bytes <= 160 KB, else PL_ERR_SHAPE.  Asynchronous on `stream`. */
int pl_simulate_runtime(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                        float inv_bandwidth, float *out_runtime, int32_t *out_events, void *stream);

/* The same with the choice of how often an output crosses the bus (appendix "Simulator", op-done
 * and transfer-done handlers).  per_child_transfers = 0 (what pl_simulate_runtime does): once per
 * destination device; its arrival releases every child waiting there.  per_child_transfers = 1:
 * the handlers as printed: the output is enqueued once for every child placed on another device
 * (children in ascending id), and the end of a transfer releases that one child; an output
 * needed by k children on one remote device then occupies the bus k times. */
int pl_simulate_runtime_ex(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                           float inv_bandwidth, int32_t per_child_transfers, float *out_runtime,
                           int32_t *out_events, void *stream);

/* The memory-penalised run time of the appendix ("Reward"): R(p) = r if m <= M, else
 * r + c (m - M), with r the simulated run time (as above), m the largest peak memory over the
 * devices and c = 2 in the paper.  The appendix says only that the start and end timestamps of
 * the operations and the tensor sizes predict the peak memory; the model used here: the output
 * of an operation occupies its device from the operation's start until the latest of its own
 * end, the end of its last consumer there and the arrival of its last outgoing transfer; on
 * every other device that consumes it a copy lives from the transfer's arrival until the end of
 * its last consumer there; intervals are half-open; a device's peak is the largest sum of live
 * output sizes (column 1 of node_feats, summed in float64) at any allocation time.
 *   mem_limit      M, in the unit of the output sizes;  mem_penalty  c (>= 0)
 *   out_reward     dev [B] fp32     R(p); NaN for a graph with a device id outside [0, D)
 *   out_runtime    dev [B] fp32     r, or NULL
 *   out_peak_mem   dev [B, D] fp32  peak of every device, or NULL
 *   out_events     dev [B] int32    as above, or NULL
 * Other arguments, limits and tie rules as pl_simulate_runtime.  The first call on a batch
 * allocates the timeline buffers ((2 + 4 D) N_tot floats); asynchronous on `stream`. */
int pl_simulate_reward(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                       float inv_bandwidth, float mem_limit, float mem_penalty, float *out_reward,
                       float *out_runtime, float *out_peak_mem, int32_t *out_events, void *stream);

/* The same with per_child_transfers as in pl_simulate_runtime_ex.  Where an output reaches a
 * device more than once, the copy there exists from its first arrival and the source is kept
 * until the last one. */
int pl_simulate_reward_ex(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                          float inv_bandwidth, int32_t per_child_transfers, float mem_limit, float mem_penalty,
                          float *out_reward, float *out_runtime, float *out_peak_mem, int32_t *out_events,
                          void *stream);

/* ---- per-stage timing, for benchmarks.  While enabled, forward and gradient calls bracket each
 * kernel stage with HIP events on the caller's stream (the BW stages are those of the reverse
 * pass: head, pooling, per-node layers at the final states, the dependent chain, projection,
 * weight gradients).  pl_profile_read synchronises those
 * events and returns, per stage, the summed milliseconds and the number of launches since
 * the last reset.  Stage ids: see pl_stage. */
typedef enum {
    PL_STAGE_PROJECT = 0, PL_STAGE_SWEEP = 1, PL_STAGE_POOL = 2, PL_STAGE_HEAD = 3,
    PL_STAGE_BW_HEAD = 4, PL_STAGE_BW_POOL = 5, PL_STAGE_BW_ACTS = 6, PL_STAGE_BW_CHAIN = 7,
    PL_STAGE_BW_PROJ = 8, PL_STAGE_BW_WGRAD = 9,
    PL_STAGE_COUNT = 10
} pl_stage;
int pl_profile_enable(pl_graph_batch *g, int32_t on);
int pl_profile_read(pl_graph_batch *g, double *ms_sum /*[PL_STAGE_COUNT]*/,
                    int64_t *launches /*[PL_STAGE_COUNT]*/, int32_t reset);

const char *pl_last_error(void);
const char *pl_version(void);

#ifdef __cplusplus
}
#endif
#endif /* PLACETO_H */
