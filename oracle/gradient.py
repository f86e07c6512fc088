"""Float64 CPU oracle for the policy gradient of one batch of decisions.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It shares no code with the HIP library and never imports it.

What it computes: the REINFORCE update of the paper's appendix ("REINFORCE Algorithm",
Eq. 1) adds, for every decision i of a rollout, grad_theta log pi_theta(a_i | s_i) times a
scalar (the return after step i minus a baseline).  For a batch of B states this module
returns

    grad = sum_b  coeff[b] * d/d theta  log softmax(logits_theta(s_b))[a_b]

with theta the flat weight blob of the policy network.  The scalars coeff[b] are inputs.
Appendix A.7 ("Entropy") adds an entropy term to the loss to encourage exploration; with a
second scalar per state, beta[b], the sum also holds beta[b] * d/d theta H(pi_theta(. | s_b)),
H(pi) = - sum_d pi_d log pi_d.

How: the forward pass of Section 2.2 / Appendix A.7 is written out once more here, node by
node in a topological order, with plain PyTorch CPU operations in float64 (the same readings
as oracle/placeto_oracle.c: residual update, ReLU after every layer of f, g, l_i, h_i, pooling
keyed by device); reverse-mode differentiation of exactly that computation is PyTorch's
autograd.  Nothing is blocked, fused or reordered.

Parity pins (tests/test_oracle_gradient.py): the logits of this forward pass equal those of the
C oracle (an independent implementation); the gradient equals central finite differences of
the C oracle's log-probability for sampled parameters of every layer; the gradient with
respect to the output bias equals coeff * (one-hot(a) - pi); linearity in coeff and
additivity over the batch.
"""
from __future__ import annotations

import numpy as np
import torch


def layer_shapes(D, H, n_layers, group_by_device):
    """(name, n_in, n_out) of every layer in blob order (matrix [in, out], then the bias)."""
    F, G = D + 4, (D if group_by_device else 1)
    out = [("proj", F, H)]
    for name in ("f_td", "g_td", "f_bu", "g_bu"):
        out += [(f"{name}.{l}", H, H) for l in range(n_layers)]
    for name in ("l_par", "l_chi", "l_pll"):
        out += [(f"{name}.{l}", 2 * H if l == 0 else H, H) for l in range(n_layers)]
    for name in ("h_par", "h_chi", "h_pll"):
        out += [(f"{name}.{l}", H, H) for l in range(n_layers)]
    out += [("pol.0", (2 + 3 * G) * H, H), ("pol.1", H, D)]
    return out


def layer_slices(D, H, n_layers, group_by_device):
    """name -> (weight slice, bias slice) into the flat blob."""
    pos, out = 0, {}
    for name, n_in, n_out in layer_shapes(D, H, n_layers, group_by_device):
        out[name] = (slice(pos, pos + n_in * n_out), slice(pos + n_in * n_out, pos + n_in * n_out + n_out))
        pos += n_in * n_out + n_out
    return out, pos


def _split(theta, D, H, n_layers, group_by_device):
    sl, total = layer_slices(D, H, n_layers, group_by_device)
    assert theta.numel() == total, "weight blob has the wrong size"
    par = {}
    for name, n_in, n_out in layer_shapes(D, H, n_layers, group_by_device):
        ws, bs = sl[name]
        par[name] = (theta[ws].reshape(n_in, n_out), theta[bs])
    return par


def _mlp(par, name, n_layers, x):
    """An embedding network: n_layers layers, ReLU after each (Appendix A.7)."""
    for l in range(n_layers):
        W, b = par[f"{name}.{l}"]
        x = torch.relu(x @ W + b)
    return x


def _topological(n, src, dst):
    par = [[] for _ in range(n)]
    chi = [[] for _ in range(n)]
    for s, d in zip(src, dst):
        chi[int(s)].append(int(d))
        par[int(d)].append(int(s))
    left = [len(p) for p in par]
    order = [v for v in range(n) if left[v] == 0]
    head = 0
    while head < len(order):
        u = order[head]
        head += 1
        for c in chi[u]:
            left[c] -= 1
            if left[c] == 0:
                order.append(c)
    if len(order) != n:
        raise ValueError("the graph has a cycle")
    return par, chi, order


def _reachable(start, nbr):
    seen = {start}
    stack = [start]
    while stack:
        u = stack.pop()
        for w in nbr[u]:
            if w not in seen:
                seen.add(w)
                stack.append(w)
    return seen


def _sweep(par, f_name, g_name, n_layers, H, order, nbr, s):
    """One pass of Section 2.2 step 2 in one direction: s_v <- s_v + g(sum_{u in xi(v)} f(s_u)),
    every neighbour final before v; an empty sum is the zero vector and still goes through g."""
    s = list(s)
    msg = [None] * len(s)
    for v in order:
        agg = torch.zeros(H, dtype=torch.float64)
        for u in nbr[v]:
            agg = agg + msg[u]
        s[v] = s[v] + _mlp(par, g_name, n_layers, agg)
        msg[v] = _mlp(par, f_name, n_layers, s[v])
    return s


def logits_graph(theta, n, src, dst, feats, placement, cur, D, H, n_layers=2, k_sweeps=1,
                 group_by_device=1, single_set=0):
    """Pre-softmax outputs [D] of the policy for one graph, as a float64 tensor that depends
    differentiably on the flat weight tensor `theta`."""
    G = D if group_by_device else 1
    par = _split(theta, D, H, n_layers, group_by_device)
    parents, children, order = _topological(n, src, dst)
    feats = np.asarray(feats, dtype=np.float64).reshape(n, 3)
    # step 1: phi_v = [time, size, one-hot(device), is-current, is-visited], projected to width H
    phi = np.zeros((n, D + 4))
    phi[:, 0], phi[:, 1] = feats[:, 0], feats[:, 1]
    phi[np.arange(n), 2 + np.asarray(placement, dtype=np.int64)] = 1.0
    phi[cur, 2 + D] = 1.0
    phi[:, 3 + D] = feats[:, 2]
    W, b = par["proj"]
    x = torch.relu(torch.from_numpy(phi) @ W + b)
    td = [x[v] for v in range(n)]
    bu = [x[v] for v in range(n)]
    # step 2
    for _ in range(k_sweeps):
        td = _sweep(par, "f_td", "g_td", n_layers, H, order, parents, td)
        bu = _sweep(par, "f_bu", "g_bu", n_layers, H, order[::-1], children, bu)
    e = [torch.cat([td[v], bu[v]]) for v in range(n)]
    # step 3: node sets of the current node, pooled per (set, device)
    up = _reachable(cur, parents)
    down = _reachable(cur, children)
    z = [e[cur]]
    for i, name in enumerate(("par", "chi", "pll")):
        P = [torch.zeros(H, dtype=torch.float64) for _ in range(G)]
        for u in range(n):
            if u == cur:
                continue
            cls = 0 if u in up else (1 if u in down else 2)
            if single_set:                  # the "simple aggregator": no partition, one set
                cls = 0
            if cls != i:
                continue
            d = int(placement[u]) if group_by_device else 0
            P[d] = P[d] + _mlp(par, f"l_{name}", n_layers, e[u])
        for d in range(G):
            z.append(_mlp(par, f"h_{name}", n_layers, P[d]))
    z = torch.cat(z)
    W1, b1 = par["pol.0"]
    W2, b2 = par["pol.1"]
    return torch.relu(z @ W1 + b1) @ W2 + b2


def entropy(logits) -> "torch.Tensor":
    """H(softmax(logits)) = - sum_d pi_d log pi_d."""
    lp = torch.log_softmax(logits, dim=0)
    return -(torch.exp(lp) * lp).sum()


def policy_gradient(n_nodes, n_edges, src, dst, feats, placement, cur, weights, actions, coeff,
                    D, H, n_layers=2, k_sweeps=1, group_by_device=1, only=None, entropy_coeff=None,
                    want_entropy=False, single_set=0):
    """grad [n_params] float64 = sum_b coeff[b] * d log pi(a_b | s_b) / d theta
    (+ entropy_coeff[b] * d H(pi(. | s_b)) / d theta when given), and logp [B] = log pi(a_b | s_b).
    `only` restricts the work to the listed graphs (the others count as zero and get logp = nan).
    With want_entropy the entropies [B] are returned as a third value."""
    n_nodes = np.asarray(n_nodes, dtype=np.int64)
    n_edges = np.asarray(n_edges, dtype=np.int64)
    B = len(n_nodes)
    noff = np.concatenate([[0], np.cumsum(n_nodes)])
    eoff = np.concatenate([[0], np.cumsum(n_edges)])
    feats = np.asarray(feats, dtype=np.float64).reshape(-1, 3)
    theta = torch.tensor(np.asarray(weights, dtype=np.float64), requires_grad=True)
    grad = np.zeros(theta.numel())
    logp = np.full(B, np.nan)
    ent = np.full(B, np.nan)
    todo = range(B) if only is None else only
    for b in todo:
        lo, hi, elo, ehi = noff[b], noff[b + 1], eoff[b], eoff[b + 1]
        logits = logits_graph(theta, int(n_nodes[b]), src[elo:ehi], dst[elo:ehi], feats[lo:hi],
                              placement[lo:hi], int(cur[b]), D, H, n_layers, k_sweeps,
                              group_by_device, single_set)
        lp = torch.log_softmax(logits, dim=0)[int(actions[b])]
        logp[b] = float(lp.detach())
        h = entropy(logits)
        ent[b] = float(h.detach())
        beta = 0.0 if entropy_coeff is None else float(entropy_coeff[b])
        if coeff[b] != 0.0 and beta == 0.0:
            (g,) = torch.autograd.grad(lp, theta)
            grad += float(coeff[b]) * g.numpy()
        elif coeff[b] != 0.0 or beta != 0.0:
            (g,) = torch.autograd.grad(float(coeff[b]) * lp + beta * h, theta)
            grad += g.numpy()
    return (grad, logp, ent) if want_entropy else (grad, logp)


def gradient_workload(w, actions, coeff, only=None, entropy_coeff=None, want_entropy=False):
    """policy_gradient on a workloads.Workload, with the weights at the precision it stores."""
    from . import weights_as_stored
    blob = weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    return policy_gradient(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst, w.node_feats, w.placement,
                           w.cur_node, blob, actions, coeff, w.D, w.H, w.n_layers, w.k_sweeps,
                           w.group_by_device, only=only, entropy_coeff=entropy_coeff,
                           want_entropy=want_entropy, single_set=getattr(w, "single_set", 0))
