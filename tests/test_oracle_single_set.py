"""Pins for the one-set pooling variant (the "simple aggregator" of the paper's comparison of
policy architectures, Section 3.3): both oracles, against facts that hold whatever the weights
are.  CPU only."""
import numpy as np
import pytest
import torch

import oracle
from oracle import gradient as og
from workloads import tiny_random_dag

D, H = 3, 8


def _case(seed, n=11, n_layers=2, k_sweeps=1, group=1):
    rng = np.random.default_rng(seed)
    src, dst = tiny_random_dag(rng, n, 0.3)
    feats = np.stack([rng.lognormal(0, 0.5, n), rng.lognormal(0, 0.5, n), (rng.random(n) < 0.5)], axis=1)
    placement = rng.integers(0, D, n).astype(np.int32)
    cur = int(rng.integers(n))
    theta = rng.normal(0, 0.35, oracle.weight_count(D, H, n_layers, group))
    return dict(n=n, src=src, dst=dst, feats=feats, placement=placement, cur=cur, theta=theta,
                n_layers=n_layers, k_sweeps=k_sweeps, group=group)


def _fwd(c, theta=None, single=0, cur=None):
    return oracle.forward_graph(c["n"], c["src"], c["dst"], c["feats"], c["placement"],
                                c["cur"] if cur is None else cur, c["theta"] if theta is None else theta,
                                D, H, c["n_layers"], c["k_sweeps"], c["group"], single_set=single)


@pytest.mark.parametrize("group", [1, 0])
def test_one_set_is_the_sum_of_the_three_when_their_networks_agree(group):
    """With l_par = l_chi = l_pll the three sums add up to the sum over every node but v*;
    the other two summaries stay empty."""
    for seed in range(4):
        c = _case(seed, group=group)
        sl, _ = og.layer_slices(D, H, 2, group)
        th = c["theta"].copy()
        for l in range(2):
            for other in ("l_chi", "l_pll"):
                for a, b in zip(sl[f"{other}.{l}"], sl[f"l_par.{l}"]):
                    th[a] = th[b]
        three = _fwd(c, th, 0)["pooled"]
        one = _fwd(c, th, 1)["pooled"]
        np.testing.assert_allclose(one[0], three.sum(axis=0), rtol=1e-12, atol=1e-13)
        assert not one[1:].any()
        assert np.abs(one[0]).max() > 1e-3
        # the node embeddings do not depend on the pooling
        np.testing.assert_array_equal(_fwd(c, th, 0)["emb"], _fwd(c, th, 1)["emb"])


def test_equal_to_the_three_sets_when_every_node_is_an_ancestor():
    """A chain read at its last node: the first set already holds every other node, so the
    variant changes nothing, logits included."""
    c = _case(5, n=9)
    c["src"] = np.arange(8, dtype=np.int32)
    c["dst"] = np.arange(1, 9, dtype=np.int32)
    a, b = _fwd(c, single=0, cur=8), _fwd(c, single=1, cur=8)
    np.testing.assert_array_equal(a["logits"], b["logits"])
    np.testing.assert_array_equal(a["pooled"], b["pooled"])
    # at the first node every other node is a descendant: the variant moves them to the first set
    a, b = _fwd(c, single=0, cur=0), _fwd(c, single=1, cur=0)
    assert not a["pooled"][0].any() and not b["pooled"][1].any()
    assert np.abs(a["logits"] - b["logits"]).max() > 1e-6


def test_no_sweeps_and_one_set_ignore_the_edges():
    """k = 0 with one set: the output is a function of the node features, the placement and v*
    alone; any two edge lists over the same nodes give the same logits."""
    c = _case(8, k_sweeps=0)
    a = _fwd(c, single=1)
    rng = np.random.default_rng(99)
    c["src"], c["dst"] = tiny_random_dag(rng, c["n"], 0.5)
    b = _fwd(c, single=1)
    np.testing.assert_allclose(a["logits"], b["logits"], rtol=1e-13, atol=1e-14)
    # with the three sets the edges matter even at k = 0
    c3 = _case(8, k_sweeps=0)
    a3 = _fwd(c3, single=0)
    c3["src"], c3["dst"] = c["src"], c["dst"]
    assert np.abs(a3["logits"] - _fwd(c3, single=0)["logits"]).max() > 1e-6


@pytest.mark.parametrize("n_layers,k_sweeps,group", [(2, 1, 1), (1, 0, 1), (2, 1, 0)])
def test_the_two_oracles_agree(n_layers, k_sweeps, group):
    for seed in range(3):
        c = _case(seed + 20, n_layers=n_layers, k_sweeps=k_sweeps, group=group)
        got = og.logits_graph(torch.tensor(c["theta"]), c["n"], c["src"], c["dst"], c["feats"], c["placement"],
                              c["cur"], D, H, n_layers, k_sweeps, group, single_set=1).numpy()
        np.testing.assert_allclose(got, _fwd(c, single=1)["logits"], rtol=1e-12, atol=1e-13)


def test_gradient_against_central_differences_and_unused_networks():
    c = _case(31)
    action = 2
    grad, logp = og.policy_gradient([c["n"]], [len(c["src"])], c["src"], c["dst"], c["feats"], c["placement"],
                                    [c["cur"]], c["theta"], [action], [1.0], D, H, single_set=1)
    assert abs(logp[0] - np.log(_fwd(c, single=1)["probs"][action])) < 1e-12
    sl, _ = og.layer_slices(D, H, 2, 1)
    rng = np.random.default_rng(2)
    h = 1e-6
    for name, (ws, bs) in sl.items():
        if name.startswith("l_chi") or name.startswith("l_pll"):
            assert not grad[ws].any() and not grad[bs].any(), name      # never applied
            continue
        for i in list(rng.choice(np.arange(ws.start, ws.stop), size=2, replace=False)) + [int(rng.integers(bs.start, bs.stop))]:
            tp, tm = c["theta"].copy(), c["theta"].copy()
            tp[i] += h
            tm[i] -= h
            fd = (np.log(_fwd(c, tp, 1)["probs"][action]) - np.log(_fwd(c, tm, 1)["probs"][action])) / (2 * h)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(grad[i])) + 2e-8, (name, i, fd, grad[i])
    assert np.abs(grad[sl["l_par.0"][0]]).max() > 1e-4
