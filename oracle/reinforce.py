"""Float64 CPU oracle for the REINFORCE accumulation (appendix "REINFORCE Algorithm", Eq. 1).

TEST INFRASTRUCTURE ONLY: imported by tests/; shares no code with the HIP library and never
imports it.

Eq. 1 updates theta by eta * sum_i grad log pi(a_i | s_i) * (sum_{i' >= i} r_i' - b_i): every
decision is weighted by the return that follows it minus a baseline, and the paper's baseline for
step i is the average of that return over the independent rollouts of the same graph under the
current policy.  This module computes those weights and, by replaying a recorded episode with
the transition of Section 2.1, the sum over all steps and rollouts of weight * grad log pi.

Readings: rollouts are grouped by an integer id given by the caller (the rollouts of one graph
share an id); a step after the end of a shorter graph's episode has reward 0 and adds nothing;
the learning rate, the optimiser and the sign convention of the reward are the caller's.
"""
from __future__ import annotations

import numpy as np

from . import episode as oe
from . import gradient as og


def returns_to_go(rewards) -> np.ndarray:
    """G[t, b] = sum over t' >= t of rewards[t', b]."""
    r = np.asarray(rewards, dtype=np.float64)
    G = np.zeros_like(r)
    for t in range(r.shape[0]):
        for u in range(t, r.shape[0]):
            G[t] += r[u]
    return G


def advantages(rewards, group, n_groups: int):
    """coeff[t, b] = G[t, b] - baseline[t, group[b]], baseline[t, g] = mean of G[t, b] over the
    rollouts b with group[b] == g (0 for an empty group; a rollout whose id is outside
    [0, n_groups) has baseline 0).  Returns (coeff [T, B], baseline [T, n_groups])."""
    G = returns_to_go(rewards)
    T, B = G.shape
    group = np.asarray(group, dtype=np.int64)
    base = np.zeros((T, n_groups))
    for g in range(n_groups):
        members = [b for b in range(B) if group[b] == g]
        if members:
            base[:, g] = G[:, members].sum(axis=1) / len(members)
    coeff = G.copy()
    for b in range(B):
        if 0 <= group[b] < n_groups:
            coeff[:, b] -= base[:, group[b]]
    return coeff, base


def episode_gradient(w, order, actions, coeff, placement0=None, entropy_coeff=None):
    """sum over steps t and rollouts b of coeff[t, b] * d log pi(actions[t, b] | s_t,b) / d theta for
    the batch of workloads.Workload `w`, every graph starting unvisited from `placement0` (default
    all on device 0) and visiting its nodes in `order` (per graph a permutation of its node ids,
    concatenated); with entropy_coeff [T, B], plus entropy_coeff[t, b] * d H(pi(. | s_t,b)) / d theta
    (Appendix A.7, "Entropy").  Returns (grad [n_params], logp [T, B] with 0 after a graph's last
    step)."""
    from . import weights_as_stored
    blob = weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    actions = np.asarray(actions)
    coeff = np.asarray(coeff, dtype=np.float64)
    T = actions.shape[0]
    grad = np.zeros(blob.size)
    logp = np.zeros((T, w.B))
    for b in range(w.B):
        n, src, dst, feats, _, _ = w.graph(b)
        n0 = int(w.node_off[b])
        ordb = np.asarray(order[n0:n0 + n])
        placement = (np.zeros(n, dtype=np.int32) if placement0 is None
                     else np.array(placement0[n0:n0 + n], dtype=np.int32, copy=True))
        f = np.array(feats, dtype=np.float64, copy=True)
        f[:, 2] = 0.0
        cur = int(ordb[0])
        for t in range(min(T, n)):
            g, lp = og.policy_gradient([n], [len(src)], src, dst, f, placement, [cur], blob,
                                       [int(actions[t, b])], [coeff[t, b]], w.D, w.H, w.n_layers,
                                       w.k_sweeps, w.group_by_device,
                                       entropy_coeff=None if entropy_coeff is None else [entropy_coeff[t, b]])
            grad += g
            logp[t, b] = lp[0]
            cur = oe.transition(placement, f[:, 2], ordb, t, cur, int(actions[t, b]))
    return grad, logp
