"""Pins for the episode oracle (oracle/episode.py, Section 2.1): closed forms and invariants
that a wrong sampler, log-probability or transition would break."""
import numpy as np
import pytest

import oracle
from oracle import episode as ep
from workloads import make_workload, make_episode


def test_uniform_logits_sample_floor_u_times_d():
    # equal logits: the cumulative distribution is (d + 1) / D, so the action is floor(u D)
    for D in (2, 4, 8):
        for u in (0.0, 0.1, 0.26, 0.5, 0.74, 0.999):
            assert ep.sample_action(np.full(D, 3.7), u) == int(np.floor(u * D))


def test_shifted_logits_give_the_same_action_and_logp():
    rng = np.random.default_rng(5)
    l = rng.normal(size=6) * 4
    for u in rng.random(20):
        assert ep.sample_action(l, u) == ep.sample_action(l + 123.0, u)
    assert abs(ep.log_prob(l, 2) - ep.log_prob(l - 50.0, 2)) < 1e-12


def test_dominant_logit_and_boundaries():
    l = np.array([0.0, 800.0, 0.0])          # no overflow: max is subtracted
    assert ep.sample_action(l, 0.5) == 1
    assert ep.sample_action(l, 0.0) == 1      # p_0 underflows to 0: not > u = 0
    l = np.log(np.array([0.25, 0.25, 0.5]))
    assert ep.sample_action(l, 0.2499) == 0
    assert ep.sample_action(l, 0.2501) == 1
    assert ep.sample_action(l, 0.75) == 2     # c_1 = 0.5 is not > 0.75; c_2 = 1 is
    assert ep.decision_margin(l, 0.26) == pytest.approx(0.01, abs=1e-12)


def test_log_probs_are_a_distribution_and_match_frequencies():
    rng = np.random.default_rng(11)
    l = rng.normal(size=5) * 2
    lp = np.array([ep.log_prob(l, a) for a in range(5)])
    assert abs(np.exp(lp).sum() - 1.0) < 1e-12
    np.testing.assert_allclose(np.exp(lp), ep.softmax(l), rtol=1e-12)
    # empirical frequencies of the sampler on a fine grid of u equal the probabilities
    us = (np.arange(20000) + 0.5) / 20000
    freq = np.bincount([ep.sample_action(l, u) for u in us], minlength=5) / 20000
    np.testing.assert_allclose(freq, ep.softmax(l), atol=1e-4)


def test_transition_and_episode_invariants():
    # Section 2.1: each step marks exactly one more node visited; the episode ends after |V|
    # steps with every node visited once, in the given order, and every placement updated.
    w = make_workload("random32")
    order, uniforms, placement0 = make_episode(w, 32)
    n = int(w.n_nodes[0])
    blob = oracle.weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    seen = []

    def fwd(placement, visited, cur):
        assert visited.sum() == len(seen)                 # one more per step
        assert visited[cur] == 0.0                        # the current node is unvisited
        seen.append(cur)
        feats = np.array(w.node_feats, dtype=np.float64)
        feats[:, 2] = visited
        return oracle.forward_graph(n, w.edge_src, w.edge_dst, feats, placement, cur, blob, w.D, w.H,
                                    w.n_layers, w.k_sweeps, w.group_by_device)["logits"]

    r = ep.run_episode(fwd, n, placement0, order[:n], uniforms[:, 0])
    assert seen == list(order[:n]) and r["cur"] == -1
    assert r["visited"].sum() == n and len(r["sampled"]) == n
    np.testing.assert_array_equal(r["placement"][order[:n]], r["sampled"])
    # replay with forced actions reproduces the trajectory and its log-probabilities
    seen.clear()
    r2 = ep.run_episode(fwd, n, placement0, order[:n], uniforms[:, 0], actions=r["sampled"])
    np.testing.assert_array_equal(r2["placement"], r["placement"])
    np.testing.assert_allclose(r2["logp"], r["logp"], rtol=0, atol=0)
    # forcing another action changes later states: the trajectory is state dependent
    forced = r["sampled"].copy()
    forced[0] = (forced[0] + 1) % w.D
    seen.clear()
    r3 = ep.run_episode(fwd, n, placement0, order[:n], uniforms[:, 0], actions=forced)
    assert not np.allclose(r3["logits"][1], r["logits"][1])
