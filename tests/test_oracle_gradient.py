"""Pins for the policy-gradient oracle (oracle/gradient.py; appendix "REINFORCE Algorithm",
Eq. 1): its forward pass against the independent C oracle, its gradient against central finite
differences of the C oracle's log-probability, closed forms and linearity.  CPU only."""
import numpy as np
import pytest

import oracle
from oracle import gradient as og
from workloads import tiny_random_dag

D, H = 3, 8


def _case(seed, n=9, n_layers=2, k_sweeps=1, group=1, D=D, H=H):
    rng = np.random.default_rng(seed)
    src, dst = tiny_random_dag(rng, n, 0.35)
    feats = np.stack([rng.lognormal(0, 0.5, n), rng.lognormal(0, 0.5, n), (rng.random(n) < 0.5)], axis=1)
    placement = rng.integers(0, D, n).astype(np.int32)
    cur = int(rng.integers(n))
    n_par = oracle.weight_count(D, H, n_layers, group)
    theta = rng.normal(0, 0.35, n_par)
    return dict(n=n, src=src, dst=dst, feats=feats, placement=placement, cur=cur, theta=theta,
                D=D, H=H, n_layers=n_layers, k_sweeps=k_sweeps, group=group)


def _c_logp(c, theta, action):
    r = oracle.forward_graph(c["n"], c["src"], c["dst"], c["feats"], c["placement"], c["cur"], theta,
                             c["D"], c["H"], c["n_layers"], c["k_sweeps"], c["group"])
    return float(np.log(r["probs"][action])), r


def _grad(c, action, coeff=1.0):
    return og.policy_gradient([c["n"]], [len(c["src"])], c["src"], c["dst"], c["feats"], c["placement"],
                              [c["cur"]], c["theta"], [action], [coeff], c["D"], c["H"], c["n_layers"],
                              c["k_sweeps"], c["group"])


@pytest.mark.parametrize("n_layers,k_sweeps,group", [(2, 1, 1), (1, 1, 1), (2, 2, 1), (2, 1, 0), (1, 0, 1), (3, 1, 1)])
def test_forward_equals_the_c_oracle(n_layers, k_sweeps, group):
    """Two implementations written separately from Section 2.2 give the same logits."""
    import torch
    for seed in range(4):
        c = _case(seed, n=11, n_layers=n_layers, k_sweeps=k_sweeps, group=group)
        got = og.logits_graph(torch.tensor(c["theta"]), c["n"], c["src"], c["dst"], c["feats"], c["placement"],
                              c["cur"], D, H, n_layers, k_sweeps, group).numpy()
        _, ref = _c_logp(c, c["theta"], 0)
        np.testing.assert_allclose(got, ref["logits"], rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n_layers,k_sweeps,group", [(2, 1, 1), (1, 1, 1), (2, 2, 1), (2, 1, 0)])
def test_gradient_equals_central_differences_of_the_c_oracle(n_layers, k_sweeps, group):
    """Sampled parameters of every layer (matrix and bias): (logp(theta + h e_i) - logp(theta - h e_i)) / 2h
    computed with the C oracle, which shares nothing with the autograd path."""
    c = _case(7, n=10, n_layers=n_layers, k_sweeps=k_sweeps, group=group)
    action = 1
    grad, logp = _grad(c, action)
    ref_lp, _ = _c_logp(c, c["theta"], action)
    assert abs(logp[0] - ref_lp) < 1e-12
    slices, total = og.layer_slices(D, H, n_layers, group)
    assert total == c["theta"].size
    rng = np.random.default_rng(0)
    h = 1e-6
    checked = 0
    for name, (ws, bs) in slices.items():
        idx = list(rng.choice(np.arange(ws.start, ws.stop), size=3, replace=False)) + [int(rng.integers(bs.start, bs.stop))]
        for i in idx:
            tp, tm = c["theta"].copy(), c["theta"].copy()
            tp[i] += h
            tm[i] -= h
            fd = (_c_logp(c, tp, action)[0] - _c_logp(c, tm, action)[0]) / (2 * h)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(grad[i])) + 2e-8, (name, i, fd, grad[i])
            checked += 1
    assert checked == 4 * len(slices)
    assert np.abs(grad).max() > 1e-3          # the case is not degenerate


def test_output_bias_gradient_is_onehot_minus_pi():
    """d log softmax(l)[a] / d l = one-hot(a) - pi, and the output bias enters l additively."""
    c = _case(3)
    for action in range(D):
        grad, _ = _grad(c, action, coeff=-2.5)
        _, ref = _c_logp(c, c["theta"], action)
        slices, _ = og.layer_slices(D, H, 2, 1)
        want = -2.5 * (np.eye(D)[action] - ref["probs"])
        np.testing.assert_allclose(grad[slices["pol.1"][1]], want, rtol=1e-12, atol=1e-14)
        assert abs(grad[slices["pol.1"][1]].sum()) < 1e-13


def test_linear_in_coeff_and_additive_over_the_batch():
    a, b = _case(11, n=7), _case(12, n=12)
    b["theta"] = a["theta"]
    ga, _ = _grad(a, 0, 1.0)
    gb, _ = _grad(b, 2, 1.0)
    both, logp = og.policy_gradient(
        [a["n"], b["n"]], [len(a["src"]), len(b["src"])], np.concatenate([a["src"], b["src"]]),
        np.concatenate([a["dst"], b["dst"]]), np.concatenate([a["feats"], b["feats"]]),
        np.concatenate([a["placement"], b["placement"]]), [a["cur"], b["cur"]], a["theta"], [0, 2], [0.5, -3.0],
        D, H)
    np.testing.assert_allclose(both, 0.5 * ga - 3.0 * gb, rtol=1e-12, atol=1e-14)
    zero, _ = og.policy_gradient(
        [a["n"], b["n"]], [len(a["src"]), len(b["src"])], np.concatenate([a["src"], b["src"]]),
        np.concatenate([a["dst"], b["dst"]]), np.concatenate([a["feats"], b["feats"]]),
        np.concatenate([a["placement"], b["placement"]]), [a["cur"], b["cur"]], a["theta"], [0, 2], [0.0, 0.0],
        D, H)
    assert not zero.any() and np.isfinite(logp).all()


def test_parameters_that_cannot_matter_get_zero_gradient():
    """A single-node graph: no messages, empty sets.  f never reaches the output, l_i is never
    applied; g (through g(0)), h_i (through h_i(0)), the projection and the policy do."""
    c = _case(5, n=1)
    c["src"], c["dst"] = np.zeros(0, np.int32), np.zeros(0, np.int32)
    grad, _ = _grad(c, 2)
    slices, _ = og.layer_slices(D, H, 2, 1)
    for name, (ws, bs) in slices.items():
        g = np.concatenate([grad[ws], grad[bs]])
        if name.startswith("f_") or name.startswith("l_"):
            assert not g.any(), name
    assert np.abs(grad[slices["pol.0"][0]]).max() > 0
    assert np.abs(grad[slices["proj"][0]]).max() > 0


def _c_entropy(c, theta):
    p = _c_logp(c, theta, 0)[1]["probs"]
    return float(-(p * np.log(p)).sum())


def test_entropy_gradient_equals_central_differences_of_the_c_oracle():
    """Appendix A.7 "Entropy": d H / d theta with H = - sum pi log pi computed from the C oracle's
    probabilities, for sampled parameters of every layer; and the value of H itself."""
    c = _case(21, n=10)
    grad, logp, ent = og.policy_gradient([c["n"]], [len(c["src"])], c["src"], c["dst"], c["feats"], c["placement"],
                                         [c["cur"]], c["theta"], [1], [0.0], D, H, entropy_coeff=[1.0],
                                         want_entropy=True)
    assert abs(ent[0] - _c_entropy(c, c["theta"])) < 1e-12
    assert 0.0 < ent[0] <= np.log(D) + 1e-12
    slices, _ = og.layer_slices(D, H, 2, 1)
    rng = np.random.default_rng(1)
    h = 1e-6
    for name, (ws, bs) in slices.items():
        for i in list(rng.choice(np.arange(ws.start, ws.stop), size=2, replace=False)) + [int(rng.integers(bs.start, bs.stop))]:
            tp, tm = c["theta"].copy(), c["theta"].copy()
            tp[i] += h
            tm[i] -= h
            fd = (_c_entropy(c, tp) - _c_entropy(c, tm)) / (2 * h)
            assert abs(fd - grad[i]) <= 1e-6 * max(1.0, abs(grad[i])) + 2e-8, (name, i, fd, grad[i])
    assert np.abs(grad).max() > 1e-4


def test_entropy_gradient_closed_form_and_mixture():
    """d H / d logits = - pi (log pi + H), through the output bias; and the two terms add."""
    c = _case(22)
    _, ref = _c_logp(c, c["theta"], 0)
    p = ref["probs"]
    Hh = -(p * np.log(p)).sum()
    slices, _ = og.layer_slices(D, H, 2, 1)
    args = ([c["n"]], [len(c["src"])], c["src"], c["dst"], c["feats"], c["placement"], [c["cur"]], c["theta"])
    g_ent, _ = og.policy_gradient(*args, [2], [0.0], D, H, entropy_coeff=[0.7])
    np.testing.assert_allclose(g_ent[slices["pol.1"][1]], 0.7 * (-p * (np.log(p) + Hh)), rtol=1e-10, atol=1e-14)
    assert abs(g_ent[slices["pol.1"][1]].sum()) < 1e-13
    g_lp, _ = og.policy_gradient(*args, [2], [-1.5], D, H)
    g_mix, _ = og.policy_gradient(*args, [2], [-1.5], D, H, entropy_coeff=[0.7])
    np.testing.assert_allclose(g_mix, g_lp + g_ent, rtol=1e-10, atol=1e-13)
    # equal logits: the entropy is at its maximum log D and its gradient vanishes
    import torch
    l = torch.zeros(D, dtype=torch.float64, requires_grad=True)
    h = og.entropy(l)
    (gl,) = torch.autograd.grad(h, l)
    assert abs(float(h) - np.log(D)) < 1e-14 and float(gl.abs().max()) < 1e-15
