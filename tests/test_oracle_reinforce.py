"""Pins for the REINFORCE accumulation oracle (oracle/reinforce.py; appendix "REINFORCE
Algorithm", Eq. 1): closed forms and invariants of the returns and baselines.  CPU only."""
import numpy as np

from oracle import reinforce as orf


def test_returns_of_constant_and_single_rewards():
    T, B = 7, 3
    G = orf.returns_to_go(np.full((T, B), 2.5))
    np.testing.assert_allclose(G[:, 0], 2.5 * (T - np.arange(T)))        # (T - t) r
    r = np.zeros((T, B))
    r[4, 1] = -3.0                                                      # one reward at step 4
    G = orf.returns_to_go(r)
    np.testing.assert_array_equal(G[:5, 1], -3.0)                        # every earlier decision sees it
    np.testing.assert_array_equal(G[5:, 1], 0.0)                         # later ones do not
    assert not G[:, [0, 2]].any()
    # terminal reward only (the paper's first reward scheme): every step's return is r_T
    r = np.zeros((T, B))
    r[-1] = [1.0, 2.0, 3.0]
    np.testing.assert_array_equal(orf.returns_to_go(r), np.tile([1.0, 2.0, 3.0], (T, 1)))


def test_returns_equal_reversed_cumulative_sum():
    rng = np.random.default_rng(0)
    r = rng.normal(size=(23, 5))
    np.testing.assert_allclose(orf.returns_to_go(r), np.cumsum(r[::-1], axis=0)[::-1], rtol=1e-12, atol=1e-12)


def test_baseline_is_the_group_mean_and_advantages_cancel():
    rng = np.random.default_rng(1)
    T, B, n_groups = 11, 9, 4
    r = rng.normal(size=(T, B))
    group = np.array([0, 1, 0, 2, 1, 0, 2, 2, 1])                       # group 3 is empty
    coeff, base = orf.advantages(r, group, n_groups)
    G = orf.returns_to_go(r)
    for g in range(3):
        np.testing.assert_allclose(base[:, g], G[:, group == g].mean(axis=1), rtol=1e-12)
        np.testing.assert_allclose(coeff[:, group == g].sum(axis=1), 0.0, atol=1e-12)   # advantages of a group cancel
    assert not base[:, 3].any()
    # identical rollouts of one graph: nothing to prefer, every weight is zero
    same = np.tile(rng.normal(size=(T, 1)), (1, 4))
    c, _ = orf.advantages(same, np.zeros(4, int), 1)
    np.testing.assert_allclose(c, 0.0, atol=1e-12)
    # a rollout alone in its group is its own baseline
    c, _ = orf.advantages(r[:, :1], [0], 1)
    np.testing.assert_allclose(c, 0.0, atol=1e-12)
    # an id outside the range keeps the plain return
    c, _ = orf.advantages(r[:, :2], [0, 7], 2)
    np.testing.assert_allclose(c[:, 1], G[:, 1])


def test_better_rollout_gets_positive_weight():
    """Two rollouts of one graph, one step: the weight is r - mean(r), positive for the better one
    (Eq. 1 raises the probability of actions whose return beats the average)."""
    c, b = orf.advantages(np.array([[1.0, 3.0]]), [0, 0], 1)
    np.testing.assert_allclose(b, [[2.0]])
    np.testing.assert_allclose(c, [[-1.0, 1.0]])
