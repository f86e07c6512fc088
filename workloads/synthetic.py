"""Seeded synthetic DAG batches, node features, episode states and weights.

The paper evaluates on TensorFlow training graphs of Inception-V3, NMT and NASNet
(Section 3, Appendix A.2) and on generated graph datasets (Appendix A.3).  None of those
graphs is reproduced here; the five recipes below only take their *shape*: fork-join
modules, unrolled recurrent chains with attention fan-in, and cells of two-input blocks,
with the gradient half of an SGD step mirrored behind the forward half where the recipe
says so.  Node features follow Section 2.1 (run time, output size, current device,
visited flag, current flag).

Nothing in this file performs the method's arithmetic.  `weight_layout` is a description
of the weight blob's interface (names and shapes in blob order), used to draw weights and
to let tests write special weights (identities, zeros) into the right slots.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED_BASE = 190608879 * 10

CONFIG_NAMES = ("random32", "layered200", "inception", "nmt", "nasnet")

# (index, B, D, H, weight_dtype)
_CONFIG_TABLE = {
    "random32": (1, 1, 2, 8, "fp32"),
    "layered200": (2, 64, 4, 32, "fp32"),
    "inception": (3, 128, 4, 64, "fp32"),
    "nmt": (4, 64, 4, 64, "fp32"),
    "nasnet": (5, 256, 8, 128, "bf16"),
}


# --------------------------------------------------------------------------- weights
def weight_layout(D: int, H: int, n_layers: int = 2, group_by_device: bool = True
                  ) -> List[Tuple[str, int, int]]:
    """Names and (in, out) shapes of every layer, in blob order.

    Each layer occupies in*out floats (row-major [in, out]) followed by `out` bias floats.
    Order: input projection; f, g top-down; f, g bottom-up; l for the parent, child and
    parallel sets; h for the same three; the two policy layers.
    """
    F = D + 4
    groups = D if group_by_device else 1
    Z = (2 + 3 * groups) * H
    out: List[Tuple[str, int, int]] = [("proj.0", F, H)]
    for name in ("f_td", "g_td", "f_bu", "g_bu"):
        for layer in range(n_layers):
            out.append((f"{name}.{layer}", H, H))
    for name in ("l_par", "l_chi", "l_pll"):
        for layer in range(n_layers):
            out.append((f"{name}.{layer}", 2 * H if layer == 0 else H, H))
    for name in ("h_par", "h_chi", "h_pll"):
        for layer in range(n_layers):
            out.append((f"{name}.{layer}", H, H))
    out.append(("policy.0", Z, H))
    out.append(("policy.1", H, D))
    return out


def weight_count(D: int, H: int, n_layers: int = 2, group_by_device: bool = True) -> int:
    return sum(i * o + o for _, i, o in weight_layout(D, H, n_layers, group_by_device))


def weight_slices(D: int, H: int, n_layers: int = 2, group_by_device: bool = True
                  ) -> Dict[str, Tuple[slice, slice, Tuple[int, int]]]:
    """name -> (matrix slice, bias slice, (in, out)) into the flat blob."""
    pos = 0
    table = {}
    for name, i, o in weight_layout(D, H, n_layers, group_by_device):
        table[name] = (slice(pos, pos + i * o), slice(pos + i * o, pos + i * o + o), (i, o))
        pos += i * o + o
    return table


# --------------------------------------------------------------------------- DAG building
class _Dag:
    """Edge-list DAG under construction; node ids are creation order (topological)."""

    def __init__(self) -> None:
        self.types: List[int] = []
        self.src: List[int] = []
        self.dst: List[int] = []
        self._seen = set()

    def node(self, op_type: int) -> int:
        self.types.append(op_type)
        return len(self.types) - 1

    def edge(self, u: int, v: int) -> bool:
        if u == v or (u, v) in self._seen:
            return False
        self._seen.add((u, v))
        self.src.append(u)
        self.dst.append(v)
        return True

    @property
    def n(self) -> int:
        return len(self.types)


def _mirror(g: _Dag, n_types: int) -> None:
    """Append the gradient half of a training step: one gradient node per forward node,
    every forward edge reversed between the gradient nodes, and forward -> gradient edges
    (the gradient of an op consumes the op's own output)."""
    n_fwd = g.n
    fwd_edges = list(zip(g.src, g.dst))
    for v in range(n_fwd):
        g.node(g.types[v] + n_types)
    for v in range(n_fwd):
        g.edge(v, n_fwd + v)
    for u, v in fwd_edges:
        g.edge(n_fwd + v, n_fwd + u)


def _dag_random32(rng: np.random.Generator) -> _Dag:
    g = _Dag()
    for i in range(32):
        g.node(0)
        if i == 0:
            continue
        n_p = int(rng.choice([1, 2, 3], p=[0.6, 0.3, 0.1]))
        for p in rng.choice(i, size=min(n_p, i), replace=False):
            g.edge(int(p), i)
    return g


def _dag_layered(rng: np.random.Generator, n_nodes: int = 200) -> _Dag:
    widths: List[int] = []
    while sum(widths) < n_nodes:
        widths.append(int(rng.integers(4, 13)))
    widths[-1] -= sum(widths) - n_nodes
    if widths[-1] == 0:
        widths.pop()
    g = _Dag()
    layers: List[List[int]] = []
    for w in widths:
        layers.append([g.node(0) for _ in range(w)])
    for li in range(1, len(layers)):
        prev = layers[li - 1]
        for v in layers[li]:
            n_p = min(1 + int(rng.binomial(2, 0.25)), len(prev))
            for p in rng.choice(len(prev), size=n_p, replace=False):
                u = prev[int(p)]
                if li >= 2 and rng.random() < 0.05:
                    far = layers[int(rng.integers(0, li - 1))]
                    u_far = far[int(rng.integers(len(far)))]
                    if g.edge(u_far, v):
                        continue
                g.edge(u, v)
    return g


# op-type ids (only used to shift the feature distributions per type)
_INC_TYPES = 8      # conv1x1, conv3x3, conv5x5, pool, act, concat, dense, loss
_NMT_TYPES = 12
_NAS_TYPES = 8


def _dag_inception(rng: np.random.Generator) -> _Dag:
    g = _Dag()
    prev = g.node(0)
    for i in range(1, 10):
        n = g.node(4 if i % 2 else 1)
        g.edge(prev, n)
        prev = n
    branch_heads: List[int] = []
    for _module in range(12):
        tails = []
        for br in range(4):
            p = prev
            for o in range(int(rng.integers(1, 5))):
                c = g.node(br)            # branch-specific compute op
                g.edge(p, c)
                a = g.node(4)             # activation
                g.edge(c, a)
                if o == 0:
                    branch_heads.append(c)
                p = a
            tails.append(p)
        cat = g.node(5)
        for t in tails:
            g.edge(t, cat)
        prev = cat
    for t in (3, 6, 6, 7):
        n = g.node(t)
        g.edge(prev, n)
        prev = n
    n_fwd = g.n
    _mirror(g, _INC_TYPES)
    for c in branch_heads:                # one weight-update node per branch
        u = g.node(2 * _INC_TYPES)
        g.edge(n_fwd + c, u)
    return g


def _lstm_cell(g: _Dag, x: int, h_prev: Optional[int], c_prev: Optional[int], base: int
               ) -> Tuple[int, int]:
    mm = g.node(base)
    g.edge(x, mm)
    if h_prev is not None:
        g.edge(h_prev, mm)
    gates = []
    for k in range(4):
        gate = g.node(base + 1)
        g.edge(mm, gate)
        gates.append(gate)
    c_new = g.node(base + 2)
    for gate in gates[:3]:
        g.edge(gate, c_new)
    if c_prev is not None:
        g.edge(c_prev, c_new)
    h_new = g.node(base + 3)
    g.edge(gates[3], h_new)
    g.edge(c_new, h_new)
    return h_new, c_new


def _dag_nmt(rng: np.random.Generator) -> _Dag:
    g = _Dag()
    t_enc = int(rng.integers(38, 43))
    t_dec = int(rng.integers(38, 43))
    n_layers = 2
    enc_h: List[List[int]] = [[] for _ in range(n_layers)]
    enc_c: List[List[int]] = [[] for _ in range(n_layers)]
    for t in range(t_enc):
        x = g.node(4)                     # source embedding lookup
        for layer in range(n_layers):
            h_prev = enc_h[layer][-1] if t else None
            c_prev = enc_c[layer][-1] if t else None
            h, c = _lstm_cell(g, x, h_prev, c_prev, 0)
            enc_h[layer].append(h)
            enc_c[layer].append(c)
            x = h
    dec_h = [enc_h[layer][-1] for layer in range(n_layers)]
    dec_c = [enc_c[layer][-1] for layer in range(n_layers)]
    losses = []
    for t in range(t_dec):
        x = g.node(5)                     # target embedding lookup
        for layer in range(n_layers):
            h, c = _lstm_cell(g, x, dec_h[layer], dec_c[layer], 0)
            dec_h[layer], dec_c[layer] = h, c
            x = h
        score = g.node(6)                 # attention scores: every encoder output + query
        for h_e in enc_h[-1]:
            g.edge(h_e, score)
        g.edge(x, score)
        soft = g.node(7)
        g.edge(score, soft)
        ctx = g.node(8)
        g.edge(soft, ctx)
        comb = g.node(9)
        g.edge(ctx, comb)
        g.edge(x, comb)
        proj = g.node(10)
        g.edge(comb, proj)
        loss = g.node(11)
        g.edge(proj, loss)
        losses.append(loss)
    total = g.node(11)
    for loss in losses:
        g.edge(loss, total)
    return g


def _dag_nasnet(rng: np.random.Generator) -> _Dag:
    g = _Dag()
    s0 = g.node(0)
    s1 = g.node(0)
    g.edge(s0, s1)
    cell_outs = [s0, s1]
    chain_heads_per_cell: List[List[int]] = []
    for _cell in range(18):
        avail = [cell_outs[-2], cell_outs[-1]]
        block_outs: List[int] = []
        used = set()
        heads: List[int] = []
        for _blk in range(5):
            ins = []
            for _op in range(2):
                cand = avail + block_outs
                s = cand[int(rng.integers(len(cand)))]
                used.add(s)
                p = s
                for j in range(8):        # relu -> depthwise -> pointwise -> bn, twice
                    n = g.node(1 + (j % 4))
                    g.edge(p, n)
                    if j == 0:
                        heads.append(n)
                    p = n
                ins.append(p)
            add = g.node(5)
            g.edge(ins[0], add)
            g.edge(ins[1], add)
            block_outs.append(add)
        cat = g.node(6)
        for b in block_outs:
            if b not in used:
                g.edge(b, cat)
        cell_outs.append(cat)
        chain_heads_per_cell.append(heads)
    prev = cell_outs[-1]
    for t in (7, 7, 7):
        n = g.node(t)
        g.edge(prev, n)
        prev = n
    n_fwd = g.n
    _mirror(g, _NAS_TYPES)
    for heads in chain_heads_per_cell:    # one weight-update node per cell
        u = g.node(2 * _NAS_TYPES)
        for h in heads:
            g.edge(n_fwd + h, u)
    return g


_BUILDERS = {
    "random32": (_dag_random32, 1),
    "layered200": (_dag_layered, 1),
    "inception": (_dag_inception, 2 * _INC_TYPES + 1),
    "nmt": (_dag_nmt, _NMT_TYPES),
    "nasnet": (_dag_nasnet, 2 * _NAS_TYPES + 1),
}


# --------------------------------------------------------------------------- workload
@dataclass
class Workload:
    """One batch of graphs with a mid-episode state and a weight blob.

    Edges are (src, dst) pairs of graph-local node ids, concatenated over graphs in batch
    order: dst consumes src's output, i.e. src is a parent of dst.  `node_feats[:, 0]` is
    the op's run time, `[:, 1]` its output size, `[:, 2]` the visited flag (Section 2.1).
    """
    name: str
    B: int
    D: int
    H: int
    n_layers: int
    k_sweeps: int
    group_by_device: int
    weight_dtype: str
    n_nodes: np.ndarray
    n_edges: np.ndarray
    edge_src: np.ndarray
    edge_dst: np.ndarray
    node_feats: np.ndarray
    placement: np.ndarray
    cur_node: np.ndarray
    weights: np.ndarray
    seed: int = 0
    single_set: int = 0       # 1: pooling over one set (every node other than the current one)
    node_off: np.ndarray = field(default=None, repr=False)
    edge_off: np.ndarray = field(default=None, repr=False)

    def __post_init__(self) -> None:
        self.node_off = np.concatenate([[0], np.cumsum(self.n_nodes)]).astype(np.int64)
        self.edge_off = np.concatenate([[0], np.cumsum(self.n_edges)]).astype(np.int64)

    @property
    def n_tot(self) -> int:
        return int(self.node_off[-1])

    @property
    def e_tot(self) -> int:
        return int(self.edge_off[-1])

    def graph(self, b: int):
        """(n, src, dst, feats, placement, cur) of graph b."""
        n0, n1 = self.node_off[b], self.node_off[b + 1]
        e0, e1 = self.edge_off[b], self.edge_off[b + 1]
        return (int(self.n_nodes[b]), self.edge_src[e0:e1], self.edge_dst[e0:e1],
                self.node_feats[n0:n1], self.placement[n0:n1], int(self.cur_node[b]))


def _draw_state(rng: np.random.Generator, n: int, D: int):
    """A mid-episode snapshot (Section 2.1): nodes are visited in an arbitrary order; the
    first t of a random order are done, the next one is the current node."""
    order = rng.permutation(n)
    t = int(rng.integers(0, n))
    done = np.zeros(n, dtype=np.float32)
    done[order[:t]] = 1.0
    placement = rng.integers(0, D, size=n).astype(np.int32)
    return placement, int(order[t]), done


def make_workload(name: str, B: Optional[int] = None, seed: Optional[int] = None,
                  D: Optional[int] = None, H: Optional[int] = None, n_layers: int = 2,
                  k_sweeps: int = 1, group_by_device: int = 1,
                  weight_dtype: Optional[str] = None, relabel: bool = True) -> Workload:
    """Build one of the five configurations (optionally with fewer graphs, for tests)."""
    idx, B0, D0, H0, wd0 = _CONFIG_TABLE[name]
    B = B0 if B is None else B
    D = D0 if D is None else D
    H = H0 if H is None else H
    weight_dtype = wd0 if weight_dtype is None else weight_dtype
    seed = SEED_BASE + idx if seed is None else seed
    builder, n_types = _BUILDERS[name]

    top = np.random.default_rng(seed)
    # per-op-type shifts of the two log-normal feature distributions (drawn once per type)
    mu_cost = top.normal(0.0, 0.5, size=n_types) if n_types > 1 else np.zeros(1)
    mu_bytes = top.normal(0.0, 0.5, size=n_types) if n_types > 1 else np.zeros(1)
    weights = top.normal(0.0, 0.1, size=weight_count(D, H, n_layers, bool(group_by_device))
                         ).astype(np.float32)

    n_nodes, n_edges, srcs, dsts, feats, places, curs = [], [], [], [], [], [], []
    for b in range(B):
        rng = np.random.default_rng([seed, b])
        g = builder(rng)
        n = g.n
        types = np.asarray(g.types, dtype=np.int64)
        src = np.asarray(g.src, dtype=np.int32)
        dst = np.asarray(g.dst, dtype=np.int32)
        if relabel:                       # node ids carry no meaning (Section 1, Section 3.3)
            perm = rng.permutation(n).astype(np.int32)      # old id -> new id
            src, dst = perm[src], perm[dst]
            new_types = np.empty_like(types)
            new_types[perm] = types
            types = new_types
            shuffle = rng.permutation(len(src))
            src, dst = src[shuffle], dst[shuffle]
        cost = np.exp(rng.normal(mu_cost[types], 1.0)).astype(np.float32)
        out_bytes = np.exp(rng.normal(10.0 + mu_bytes[types], 1.0)).astype(np.float32)
        placement, cur, done = _draw_state(rng, n, D)
        n_nodes.append(n)
        n_edges.append(len(src))
        srcs.append(src)
        dsts.append(dst)
        feats.append(np.stack([cost, out_bytes, done], axis=1))
        places.append(placement)
        curs.append(cur)

    return Workload(
        name=name, B=B, D=D, H=H, n_layers=n_layers, k_sweeps=k_sweeps,
        group_by_device=group_by_device, weight_dtype=weight_dtype,
        n_nodes=np.asarray(n_nodes, dtype=np.int32),
        n_edges=np.asarray(n_edges, dtype=np.int32),
        edge_src=np.concatenate(srcs).astype(np.int32) if srcs else np.zeros(0, np.int32),
        edge_dst=np.concatenate(dsts).astype(np.int32) if dsts else np.zeros(0, np.int32),
        node_feats=np.concatenate(feats).astype(np.float32),
        placement=np.concatenate(places).astype(np.int32),
        cur_node=np.asarray(curs, dtype=np.int32),
        weights=weights, seed=seed)


def make_states(w: Workload, n_states: int, seed: Optional[int] = None):
    """An episode-like stream of states for a workload's graphs.

    Returns (placement [S, N_tot] int32, cur_node [S, B] int32, done [S, N_tot] float32).
    """
    seed = w.seed + 7919 if seed is None else seed
    placement = np.empty((n_states, w.n_tot), dtype=np.int32)
    cur = np.empty((n_states, w.B), dtype=np.int32)
    done = np.empty((n_states, w.n_tot), dtype=np.float32)
    for s in range(n_states):
        rng = np.random.default_rng([seed, s])
        for b in range(w.B):
            n0, n1 = w.node_off[b], w.node_off[b + 1]
            p, c, d = _draw_state(rng, int(n1 - n0), w.D)
            placement[s, n0:n1] = p
            cur[s, b] = c
            done[s, n0:n1] = d
    return placement, cur, done


def make_episode(w: Workload, n_steps: int, seed: Optional[int] = None):
    """Inputs of an on-device episode: a visiting order per graph (a permutation of its
    graph-local node ids, concatenated), uniform numbers in [0, 1) for the sampled actions
    [n_steps, B] (float32), and the trivial start placement (every node on device 0).
    """
    seed = w.seed + 104729 if seed is None else seed
    rng = np.random.default_rng([seed, n_steps])
    order = np.empty(w.n_tot, dtype=np.int32)
    for b in range(w.B):
        n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
        order[n0:n1] = rng.permutation(n1 - n0).astype(np.int32)
    uniforms = rng.random((n_steps, w.B), dtype=np.float32)
    placement0 = np.zeros(w.n_tot, dtype=np.int32)
    return order, uniforms, placement0


def tiny_random_dag(rng: np.random.Generator, n: int, p_edge: float = 0.35):
    """A random DAG on n nodes with shuffled labels (for brute-force tests)."""
    order = rng.permutation(n)
    src, dst = [], []
    for i in range(n):
        for j in range(i + 1, n):
            if rng.random() < p_edge:
                src.append(int(order[i]))
                dst.append(int(order[j]))
    return np.asarray(src, dtype=np.int32), np.asarray(dst, dtype=np.int32)
