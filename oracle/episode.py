"""Float64 CPU oracle for one MDP transition and a whole episode (Section 2.1).

TEST INFRASTRUCTURE ONLY: imported by tests/ and the smoke check; shares no code with the
HIP library and never imports it.

Section 2.1: at step t the agent picks a device for the current node v of state s_t; in
s_{t+1} the node carries the new device, is marked visited, and an unvisited node becomes
the current node; an episode ends after |V| steps, when every node has been visited.  The
policy is the softmax over the D logits of the forward pass (Appendix A.7).

Readings (the paper fixes neither): the visiting order is an input (any permutation of the
graph's nodes); an action is drawn from the softmax by inverse CDF over devices 0..D-1 with
a uniform number u in [0, 1) that is an input as well: the first device whose cumulative
probability exceeds u, the last device if rounding leaves none.
"""
from __future__ import annotations

import numpy as np


def softmax(logits) -> np.ndarray:
    """exp(l - max) / sum, in float64 (Appendix A.7: softmax output layer)."""
    l = np.asarray(logits, dtype=np.float64)
    e = np.exp(l - l.max())
    return e / e.sum()


def sample_action(logits, u: float) -> int:
    """Inverse CDF: the first device d with p_0 + ... + p_d > u."""
    p = softmax(logits)
    c = 0.0
    for d in range(len(p)):
        c += p[d]
        if c > u:
            return d
    return len(p) - 1


def decision_margin(logits, u: float) -> float:
    """Distance of u from the nearest boundary of the cumulative distribution: a sampler in
    another precision may legitimately pick the neighbouring device when this is tiny."""
    c = np.cumsum(softmax(logits))
    return float(np.min(np.abs(c[:-1] - u))) if len(c) > 1 else 1.0


def log_prob(logits, a: int) -> float:
    """log pi(a | s) = l_a - max - log sum exp(l - max)."""
    l = np.asarray(logits, dtype=np.float64)
    m = l.max()
    return float(l[a] - m - np.log(np.exp(l - m).sum()))


def transition(placement, visited, order, t: int, cur: int, action: int):
    """s_t -> s_{t+1} for one graph, in place: the current node takes the device, is marked
    visited, and the next node of the visiting order becomes current (-1 after the last).
    Returns the new current node."""
    placement[cur] = action
    visited[cur] = 1.0
    return int(order[t + 1]) if t + 1 < len(order) else -1


def run_episode(forward_graph, n: int, placement0, order, uniforms, actions=None):
    """A whole episode of one graph.  forward_graph(placement, visited, cur) -> logits [D].
    `actions`, when given, replaces the sampled actions (replay of a recorded trajectory);
    sampled ones are still returned so that the two can be compared.
    Returns dict(logits [T, D], sampled [T], margin [T], logp [T] of the action taken,
    placement [n], visited [n])."""
    placement = np.array(placement0, dtype=np.int32, copy=True)
    visited = np.zeros(n, dtype=np.float64)
    cur = int(order[0])
    T = len(uniforms)
    out_l, out_a, out_m, out_lp = [], [], [], []
    for t in range(T):
        if cur < 0:
            break
        logits = np.asarray(forward_graph(placement, visited, cur), dtype=np.float64)
        a = sample_action(logits, float(uniforms[t]))
        taken = a if actions is None else int(actions[t])
        out_l.append(logits)
        out_a.append(a)
        out_m.append(decision_margin(logits, float(uniforms[t])))
        out_lp.append(log_prob(logits, taken))
        cur = transition(placement, visited, order, t, cur, taken)
    return dict(logits=np.array(out_l), sampled=np.array(out_a, dtype=np.int32),
                margin=np.array(out_m), logp=np.array(out_lp), placement=placement,
                visited=visited, cur=cur)
