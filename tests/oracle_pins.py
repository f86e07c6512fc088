"""Pins for the float64 oracle: each function checks it against something the paper or the
mathematics fixes (hand-derived fixtures, closed forms, library routines on special cases,
brute force, invariants) and raises AssertionError when the oracle disagrees.

Every pin takes the loaded oracle library as `lib`, so that the same checks can be run
against deliberately broken copies of the oracle (tests/test_oracle_mutations.py).
"""
from __future__ import annotations

import itertools
import os

import numpy as np

import oracle
from workloads import make_workload, tiny_random_dag, weight_count
from workloads.synthetic import weight_slices

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
TOL = dict(rtol=1e-12, atol=1e-12)


# ----------------------------------------------------------------------------- helpers
def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, vals = line.split(":", 1)
            out[key.strip()] = np.array([float(t) for t in vals.split()])
    return out


def blob(D, H, n_layers, group, layers):
    """Flat weight blob from {layer name: (W [in,out], bias [out])}; missing layers are 0."""
    table = weight_slices(D, H, n_layers, bool(group))
    w = np.zeros(weight_count(D, H, n_layers, bool(group)), dtype=np.float64)
    for name, (W, b) in layers.items():
        ms, bs, shape = table[name]
        W = np.asarray(W, dtype=np.float64)
        assert W.shape == shape, (name, W.shape, shape)
        w[ms] = W.reshape(-1)
        w[bs] = np.asarray(b, dtype=np.float64)
    return w


def identity_layers(D, n_layers=1):
    """All embedding networks = identity on H = F = D + 4 (l_i adds the two halves)."""
    H = D + 4
    eye, zero = np.eye(H), np.zeros(H)
    layers = {"proj.0": (eye, zero)}
    for name in ("f_td", "g_td", "f_bu", "g_bu", "h_par", "h_chi", "h_pll"):
        for l in range(n_layers):
            layers[f"{name}.{l}"] = (eye, zero)
    for name in ("l_par", "l_chi", "l_pll"):
        layers[f"{name}.0"] = (np.vstack([eye, eye]), zero)
        for l in range(1, n_layers):
            layers[f"{name}.{l}"] = (eye, zero)
    return layers


def random_blob(rng, D, H, n_layers=2, group=1, scale=0.5):
    return rng.normal(0.0, scale, size=weight_count(D, H, n_layers, bool(group)))


def random_state(rng, n, D):
    feats = np.stack([rng.lognormal(0, 1, n), rng.lognormal(0, 1, n),
                      (rng.random(n) < 0.5).astype(float)], axis=1)
    return feats, rng.integers(0, D, n).astype(np.int32), int(rng.integers(n))


def raw_features(feats, placement, cur, D):
    """[time, size, one-hot device, is-current, is-visited] (Section 2.1)."""
    n = len(placement)
    phi = np.zeros((n, D + 4))
    phi[:, 0:2] = feats[:, 0:2]
    phi[np.arange(n), 2 + np.asarray(placement)] = 1.0
    phi[cur, 2 + D] = 1.0
    phi[:, 3 + D] = feats[:, 2]
    return phi


def adjacency(n, src, dst):
    A = np.zeros((n, n))
    A[np.asarray(src, dtype=int), np.asarray(dst, dtype=int)] = 1.0
    return A


def closure(n, src, dst):
    """reach[u, v] = there is a non-empty path u ~> v (Warshall's algorithm)."""
    reach = adjacency(n, src, dst) > 0
    for k in range(n):
        reach |= np.outer(reach[:, k], reach[k, :])
    return reach


def fwd(lib, n, src, dst, feats, placement, cur, w, D, H, **kw):
    return oracle.forward_graph(n, src, dst, feats, placement, cur, w, D, H, lib=lib, **kw)


# ----------------------------------------------------------------------------- fixtures
_TWO_NODE = {
    "proj.0": ([[1, 0], [0, 1], [1, -1], [0, 2], [2, 1], [-1, 1]], [0, -1]),
    "f_td.0": ([[1, 2], [0, 1]], [0, 0]),
    "g_td.0": ([[0, 1], [1, 1]], [1, -2]),
    "f_bu.0": ([[1, 0], [1, 1]], [0, 1]),
    "g_bu.0": ([[2, 0], [-1, 1]], [0, 0]),
    "l_par.0": ([[1, 0], [0, 1], [1, 1], [0, -1]], [0, 0]),
    "l_chi.0": ([[1, 0], [0, 0], [0, 2], [1, 1]], [0, -3]),
    "l_pll.0": ([[0, 1], [1, 0], [0, 0], [2, 0]], [-1, 0]),
    "h_par.0": ([[1, -1], [0, 1]], [0, 1]),
    "h_chi.0": ([[1, 1], [0, -1]], [2, 0]),
    "h_pll.0": ([[0, 1], [1, 0]], [0, 0]),
    "policy.1": ([[0.1, 0.2], [0.5, 0.0]], [0, -1]),
}


def pin_two_node_asymmetric(lib):
    """tests/golden/two_node_asymmetric.txt: hand-derived, asymmetric integer weights."""
    gold = read_golden("two_node_asymmetric.txt")
    W1 = np.zeros((16, 2))
    W1[[0, 5, 8, 15], 0] = 1.0
    W1[1, 1], W1[6, 1], W1[14, 1] = 1.0, -1.0, 1.0
    layers = dict(_TWO_NODE)
    layers["policy.0"] = (W1, [-10, 3])
    w = blob(2, 2, 1, 1, layers)
    for case in ("case1", "case2"):
        r = fwd(lib, 3, [0], [1], gold[f"{case}.feats"].reshape(3, 3),
                gold[f"{case}.placement"].astype(np.int32), int(gold[f"{case}.cur"][0]), w,
                2, 2, n_layers=1)
        np.testing.assert_allclose(r["emb"].reshape(-1), gold[f"{case}.emb"], **TOL)
        np.testing.assert_allclose(r["pooled"].reshape(-1), gold[f"{case}.pooled"], **TOL)
        np.testing.assert_allclose(r["logits"], gold[f"{case}.logits"], **TOL)
        np.testing.assert_allclose(r["probs"], gold[f"{case}.probs"], **TOL)


def pin_chain3(lib):
    """tests/golden/chain3_identity.txt."""
    gold = read_golden("chain3_identity.txt")
    D, H = 2, 6
    layers = identity_layers(D)
    Z = (2 + 3 * D) * H
    W2 = np.zeros((H, D))
    W2[0] = [1.0, 2.0]
    layers["policy.0"] = (np.full((Z, H), 0.01), np.zeros(H))
    layers["policy.1"] = (W2, np.zeros(D))
    w = blob(D, H, 1, 1, layers)
    e = gold["edges"].astype(np.int32).reshape(-1, 2)
    r = fwd(lib, 3, e[:, 0], e[:, 1], gold["feats"].reshape(3, 3),
            gold["placement"].astype(np.int32), int(gold["cur"][0]), w, D, H, n_layers=1)
    np.testing.assert_allclose(r["emb"].reshape(-1), gold["emb"], **TOL)
    np.testing.assert_allclose(r["pooled"].reshape(-1), gold["pooled"], **TOL)
    np.testing.assert_allclose(r["logits"], gold["logits"], **TOL)
    np.testing.assert_allclose(r["probs"], gold["probs"], **TOL)


def pin_diamond(lib):
    """tests/golden/diamond_identity.txt: path multiplicity 2 and the three sets."""
    gold = read_golden("diamond_identity.txt")
    D, H = 2, 6
    w = blob(D, H, 1, 1, identity_layers(D))
    e = gold["edges"].astype(np.int32).reshape(-1, 2)
    r = fwd(lib, 4, e[:, 0], e[:, 1], gold["feats"].reshape(4, 3),
            gold["placement"].astype(np.int32), int(gold["cur"][0]), w, D, H, n_layers=1)
    np.testing.assert_allclose(r["emb"].reshape(-1), gold["emb"], **TOL)
    for cur, key in ((1, "classes_cur1"), (0, "classes_cur0")):
        cls = oracle.classes(4, e[:, 0], e[:, 1], cur, lib=lib)
        np.testing.assert_array_equal(cls, gold[key].astype(np.uint8))


# ----------------------------------------------------------------------------- closed forms
def pin_path_count_closed_form(lib):
    """Identity networks, non-negative features: k sweeps give td = (I - A^T)^-k phi and
    bu = (I - A)^-k phi, i.e. path-count weighted sums (Section 2.2 step 2)."""
    rng = np.random.default_rng(11)
    for trial in range(20):
        n = int(rng.integers(2, 13))
        D = int(rng.integers(1, 4))
        H = D + 4
        src, dst = tiny_random_dag(rng, n, 0.4)
        feats, placement, cur = random_state(rng, n, D)
        k = 1 + trial % 3
        n_layers = 1 + trial % 2
        w = blob(D, H, n_layers, 1, identity_layers(D, n_layers))
        r = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=n_layers, k_sweeps=k)
        phi = raw_features(feats, placement, cur, D)
        A = adjacency(n, src, dst)
        td, bu = phi, phi
        for _ in range(k):
            td = np.linalg.solve(np.eye(n) - A.T, td)
            bu = np.linalg.solve(np.eye(n) - A, bu)
        np.testing.assert_allclose(r["emb"][:, :H], td, rtol=1e-10, atol=1e-10)
        np.testing.assert_allclose(r["emb"][:, H:], bu, rtol=1e-10, atol=1e-10)
        # pooling with l = [I;I], h = I: sum of td+bu over each (set, device) group
        reach = closure(n, src, dst)
        P = np.zeros((3, D, H))
        for u in range(n):
            if u == cur:
                continue
            i = 0 if reach[u, cur] else (1 if reach[cur, u] else 2)
            P[i, placement[u]] += td[u] + bu[u]
        np.testing.assert_allclose(r["pooled"], P, rtol=1e-10, atol=1e-10)


def _torch_mlp(x, table, w, name, n_layers):
    import torch
    import torch.nn.functional as Fn
    for l in range(n_layers):
        ms, bs, shape = table[f"{name}.{l}"]
        W = torch.tensor(w[ms].reshape(shape))
        x = torch.relu(Fn.linear(x, W.T, torch.tensor(w[bs])))
    return x


def pin_two_node_path_feedforward(lib):
    """On the path a -> b with b current, and on a single node, the whole policy is a plain
    feed-forward composition; evaluate that with torch.nn.functional.linear in float64."""
    import torch
    import torch.nn.functional as Fn
    rng = np.random.default_rng(5)
    for trial in range(6):
        D, H, L = (2, 5, 2) if trial % 2 else (3, 4, 1 + trial % 3)
        G = D
        w = random_blob(rng, D, H, L)
        table = weight_slices(D, H, L, True)
        n = 1 if trial >= 4 else 2
        feats, placement, _ = random_state(rng, n, D)
        cur = n - 1
        src, dst = ([0], [1]) if n == 2 else ([], [])
        r = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L)
        phi = torch.tensor(raw_features(feats, placement, cur, D))
        x = _torch_mlp(phi, table, w, "proj", 1)
        zero = torch.zeros(H, dtype=torch.float64)
        mlp = lambda v, name: _torch_mlp(v, table, w, name, L)
        if n == 2:
            td_a = x[0] + mlp(zero, "g_td")
            td_b = x[1] + mlp(mlp(td_a, "f_td"), "g_td")
            bu_b = x[1] + mlp(zero, "g_bu")
            bu_a = x[0] + mlp(mlp(bu_b, "f_bu"), "g_bu")
            emb = torch.stack([torch.cat([td_a, bu_a]), torch.cat([td_b, bu_b])])
            P = torch.zeros(3, G, H, dtype=torch.float64)
            P[0, placement[0]] = mlp(emb[0], "l_par")
        else:
            emb = torch.cat([x[0] + mlp(zero, "g_td"), x[0] + mlp(zero, "g_bu")])[None]
            P = torch.zeros(3, G, H, dtype=torch.float64)
        q = [mlp(P[i, d], ("h_par", "h_chi", "h_pll")[i]) for i in range(3) for d in range(G)]
        z = torch.cat([emb[cur]] + q)
        ms, bs, shape = table["policy.0"]
        hid = torch.relu(Fn.linear(z, torch.tensor(w[ms].reshape(shape)).T, torch.tensor(w[bs])))
        ms, bs, shape = table["policy.1"]
        logits = Fn.linear(hid, torch.tensor(w[ms].reshape(shape)).T, torch.tensor(w[bs]))
        np.testing.assert_allclose(r["emb"], emb.numpy(), rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(r["pooled"], P.numpy(), rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(r["logits"], logits.numpy(), rtol=1e-11, atol=1e-11)
        np.testing.assert_allclose(r["probs"], torch.softmax(logits, 0).numpy(),
                                   rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------- invariants
def _random_case(rng, n=None, D=None, H=None, L=2):
    n = int(rng.integers(3, 14)) if n is None else n
    D = int(rng.integers(2, 5)) if D is None else D
    H = int(rng.integers(3, 9)) if H is None else H
    src, dst = tiny_random_dag(rng, n, 0.35)
    feats, placement, cur = random_state(rng, n, D)
    return n, D, H, L, src, dst, feats, placement, cur, random_blob(rng, D, H, L)


def pin_relabel_invariance(lib):
    """The policy must not depend on an arbitrary labelling of the nodes (Section 1 and
    Section 3.3): permuting node ids permutes the embeddings and leaves the logits alone."""
    rng = np.random.default_rng(21)
    for _ in range(10):
        n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
        r0 = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L)
        perm = rng.permutation(n)                       # old id -> new id
        inv = np.argsort(perm)
        r1 = fwd(lib, n, perm[src], perm[dst], feats[inv], placement[inv], int(perm[cur]), w,
                 D, H, n_layers=L)
        np.testing.assert_allclose(r1["logits"], r0["logits"], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r1["emb"][perm], r0["emb"], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r1["pooled"], r0["pooled"], rtol=1e-11, atol=1e-12)


def pin_edge_order_independence(lib):
    """Aggregations are plain sums (Section 2.2 steps 2-3): the order in which edges are
    listed cannot matter."""
    rng = np.random.default_rng(22)
    for _ in range(10):
        n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
        r0 = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L)
        sh = rng.permutation(len(src))
        r1 = fwd(lib, n, src[sh], dst[sh], feats, placement, cur, w, D, H, n_layers=L)
        np.testing.assert_allclose(r1["logits"], r0["logits"], rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(r1["emb"], r0["emb"], rtol=1e-11, atol=1e-12)


def pin_locality(lib):
    """The top-down summary of v covers exactly the sub-graph that can reach v, the
    bottom-up one the sub-graph reachable from v (Section 2.2 step 2): perturbing node u's
    features changes td_v only if u = v or u ~> v, and bu_v only if u = v or v ~> u."""
    rng = np.random.default_rng(23)
    changed_somewhere = False
    for _ in range(12):
        n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
        # strictly positive networks so that a perturbation is never clipped away by a ReLU
        w = np.abs(w) + 0.01
        reach = closure(n, src, dst)
        r0 = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L)
        u = int(rng.integers(n))
        feats2 = feats.copy()
        feats2[u, 0] += 1.0
        r1 = fwd(lib, n, src, dst, feats2, placement, cur, w, D, H, n_layers=L)
        for v in range(n):
            td_same = np.array_equal(r0["emb"][v, :H], r1["emb"][v, :H])
            bu_same = np.array_equal(r0["emb"][v, H:], r1["emb"][v, H:])
            assert td_same == (not (u == v or reach[u, v])), ("td", u, v)
            assert bu_same == (not (u == v or reach[v, u])), ("bu", u, v)
            changed_somewhere |= not td_same
    assert changed_somewhere


def pin_pooling_groups(lib):
    """Device-keyed pooling refines the printed per-set pooling: summing P[i][d] over
    devices gives the ungrouped P[i]; devices holding no node of a set pool to zero."""
    rng = np.random.default_rng(24)
    for _ in range(8):
        n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
        table_g = weight_slices(D, H, L, True)
        table_u = weight_slices(D, H, L, False)
        w_u = np.zeros(weight_count(D, H, L, False))
        for name in table_u:
            if name != "policy.0":
                w_u[table_u[name][0]] = w[table_g[name][0]]
                w_u[table_u[name][1]] = w[table_g[name][1]]
        rg = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L)
        ru = fwd(lib, n, src, dst, feats, placement, cur, w_u, D, H, n_layers=L, group_by_device=0)
        np.testing.assert_allclose(rg["pooled"].sum(axis=1), ru["pooled"][:, 0], rtol=1e-11, atol=1e-12)
        cls = oracle.classes(n, src, dst, cur, lib=lib)
        for i in range(3):
            for d in range(D):
                if not np.any((cls == i + 1) & (placement == d)):
                    assert np.all(rg["pooled"][i, d] == 0.0)
        one = np.full(n, D - 1, dtype=np.int32)
        r1 = fwd(lib, n, src, dst, feats, one, cur, w, D, H, n_layers=L)
        assert np.all(r1["pooled"][:, : D - 1] == 0.0)


def pin_zero_sweeps(lib):
    """k = 0 removes the neighbourhood summarisation (the 'simple partitioner' ablation of
    Section 3.3): every embedding is [x_v ; x_v] with x_v the projected raw features."""
    rng = np.random.default_rng(25)
    n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
    r = fwd(lib, n, src, dst, feats, placement, cur, w, D, H, n_layers=L, k_sweeps=0)
    table = weight_slices(D, H, L, True)
    ms, bs, shape = table["proj.0"]
    x = np.maximum(raw_features(feats, placement, cur, D) @ w[ms].reshape(shape) + w[bs], 0.0)
    np.testing.assert_allclose(r["emb"][:, :H], x, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r["emb"][:, H:], x, rtol=1e-12, atol=1e-12)


def pin_batching(lib):
    """Graphs in a batch are independent: copies give identical rows, and a graph's result
    does not depend on its batch-mates."""
    rng = np.random.default_rng(26)
    cases = [_random_case(rng, D=3, H=5) for _ in range(3)]
    w = cases[0][-1]
    singles = [fwd(lib, c[0], c[4], c[5], c[6], c[7], c[8], w, 3, 5, n_layers=2) for c in cases]
    order = [0, 1, 0, 2, 0]
    args = dict(
        n_nodes=[cases[i][0] for i in order], n_edges=[len(cases[i][4]) for i in order],
        src=np.concatenate([cases[i][4] for i in order]),
        dst=np.concatenate([cases[i][5] for i in order]),
        feats=np.concatenate([cases[i][6] for i in order]),
        placement=np.concatenate([cases[i][7] for i in order]),
        cur=[cases[i][8] for i in order])
    rb = oracle.forward_batch(weights=w, D=3, H=5, n_layers=2, n_threads=2, lib=lib, **args)
    for row, i in enumerate(order):
        np.testing.assert_array_equal(rb["logits"][row], singles[i]["logits"])
        np.testing.assert_array_equal(rb["pooled"][row], singles[i]["pooled"])
    np.testing.assert_array_equal(rb["emb"][: cases[0][0]], singles[0]["emb"])


def pin_softmax(lib):
    """The output layer is a softmax over devices (Appendix A.7)."""
    from scipy.special import softmax
    rng = np.random.default_rng(27)
    for scale in (0.3, 3.0, 30.0):
        n, D, H, L, src, dst, feats, placement, cur, w = _random_case(rng)
        r = fwd(lib, n, src, dst, feats, placement, cur, w * scale, D, H, n_layers=L)
        assert np.all(r["probs"] >= 0) and abs(r["probs"].sum() - 1.0) < 1e-12
        np.testing.assert_allclose(r["probs"], softmax(r["logits"]), rtol=1e-11, atol=1e-300)


# ----------------------------------------------------------------------------- structure
def _longest_path_to(v, parents):
    """Length of the longest path ending in v, by exhaustive recursion (tiny graphs only)."""
    return 0 if not parents[v] else 1 + max(_longest_path_to(u, parents) for u in parents[v])


def pin_levels_bruteforce(lib):
    rng = np.random.default_rng(31)
    for _ in range(60):
        n = int(rng.integers(1, 9))
        src, dst = tiny_random_dag(rng, n, 0.4)
        parents = [[int(s) for s, d in zip(src, dst) if d == v] for v in range(n)]
        children = [[int(d) for s, d in zip(src, dst) if s == v] for v in range(n)]
        td, bu = oracle.levels(n, src, dst, lib=lib)
        np.testing.assert_array_equal(td, [_longest_path_to(v, parents) for v in range(n)])
        np.testing.assert_array_equal(bu, [_longest_path_to(v, children) for v in range(n)])


def pin_level_invariants(lib):
    for name in ("random32", "layered200", "inception", "nmt", "nasnet"):
        w = make_workload(name, B=2)
        for b in range(w.B):
            n, src, dst, *_ = w.graph(b)
            td, bu = oracle.levels(n, src, dst, lib=lib)
            assert np.all(td[src] < td[dst]) and np.all(bu[src] > bu[dst])
            has_parent = np.zeros(n, bool)
            has_parent[dst] = True
            has_child = np.zeros(n, bool)
            has_child[src] = True
            np.testing.assert_array_equal(td == 0, ~has_parent)
            np.testing.assert_array_equal(bu == 0, ~has_child)
            assert td.max() == bu.max()
            # every non-root has a parent exactly one level up (longest path is tight)
            best = np.full(n, -1)
            np.maximum.at(best, dst, td[src])
            np.testing.assert_array_equal(td[has_parent], best[has_parent] + 1)


def pin_classes_closure(lib):
    """S_parents / S_children / S_parallel by boolean transitive closure (Section 2.2
    step 3), on many tiny DAGs and every choice of current node."""
    rng = np.random.default_rng(32)
    for _ in range(300):
        n = int(rng.integers(1, 8))
        src, dst = tiny_random_dag(rng, n, float(rng.uniform(0.1, 0.7)))
        reach = closure(n, src, dst)
        for cur in range(n):
            cls = oracle.classes(n, src, dst, cur, lib=lib)
            want = np.where(np.arange(n) == cur, 0,
                            np.where(reach[:, cur], 1, np.where(reach[cur, :], 2, 3)))
            np.testing.assert_array_equal(cls, want)
            rev = oracle.classes(n, dst, src, cur, lib=lib)       # reversed graph swaps 1 <-> 2
            np.testing.assert_array_equal(rev, np.array([0, 2, 1, 3])[want])


ALL_PINS = [
    pin_two_node_asymmetric, pin_chain3, pin_diamond, pin_path_count_closed_form,
    pin_two_node_path_feedforward, pin_relabel_invariance, pin_edge_order_independence,
    pin_locality, pin_pooling_groups, pin_zero_sweeps, pin_batching, pin_softmax,
    pin_levels_bruteforce, pin_level_invariants, pin_classes_closure,
]
