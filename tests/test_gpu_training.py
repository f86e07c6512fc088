"""The pieces compose into the paper's training loop (Section 2.1 episode, appendix simulator,
appendix "REINFORCE Algorithm" Eq. 1, Adam as in Appendix A.7), all through the C ABI: rollouts
on the device, simulated run times as the terminal reward, return-minus-baseline weights, the
policy gradient by replay; only the optimiser step runs on the host.  On a graph whose transfers
cost five times an operation the best placement has a closed form - everything on one device, run
time = the sum of the costs - and a randomly initialised policy must find it."""
import numpy as np
import pytest

from workloads import tiny_random_dag, weight_count

pytestmark = pytest.mark.gpu


def test_policy_learns_to_colocate_when_transfers_dominate():
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(0)
    n, D, H, R = 14, 3, 16, 32                       # one graph, 32 rollouts per iteration
    src, dst = tiny_random_dag(rng, n, 0.25)
    feats0 = np.tile(np.stack([np.ones(n), np.ones(n), np.zeros(n)], axis=1).astype(np.float32), (R, 1))
    g = pl.GraphBatch(np.full(R, n, np.int32), np.full(R, len(src), np.int32), np.tile(src, R), np.tile(dst, R))
    order = torch.from_numpy(np.tile(np.arange(n, dtype=np.int32), R)).to(dev)
    group = torch.zeros(R, dtype=torch.int32, device=dev)
    n_par = weight_count(D, H, 2, True)
    theta = rng.normal(0, 0.1, n_par).astype(np.float32)
    m, v = np.zeros_like(theta), np.zeros_like(theta)
    inv_bw, lr, iters = 5.0, 0.02, 25
    history = []
    for it in range(iters):
        wt = pl.Weights(theta, D, H, 2, 1, 1, "fp32")
        start = torch.from_numpy(rng.integers(0, D, R * n).astype(np.int32)).to(dev)   # arbitrary initial placement
        f, p, c = torch.from_numpy(feats0.copy()).to(dev), start.clone(), torch.zeros(R, dtype=torch.int32, device=dev)
        u = torch.from_numpy(rng.random((n, R), dtype=np.float32)).to(dev)
        logits = torch.empty((R, D), dtype=torch.float32, device=dev)
        actions = torch.empty((n, R), dtype=torch.int32, device=dev)
        pl.episode_run(g, wt, f, p, c, order, u, 0, n, logits, False, actions)
        runtime = torch.empty(R, dtype=torch.float32, device=dev)
        pl.simulate_runtime(g, D, f, p, inv_bw, runtime)
        rewards = torch.zeros((n, R), dtype=torch.float32, device=dev)
        rewards[-1] = -runtime                                         # terminal reward (Appendix A.7)
        coeff = torch.empty((n, R), dtype=torch.float32, device=dev)
        baseline = torch.empty((n, 1), dtype=torch.float32, device=dev)
        pl.reinforce_coeff(rewards, group, 1, coeff, baseline)
        f2, c2 = torch.from_numpy(feats0.copy()).to(dev), torch.zeros(R, dtype=torch.int32, device=dev)
        grad = torch.empty(n_par, dtype=torch.float32, device=dev)
        pl.episode_gradient(g, wt, f2, start, c2, order, actions, coeff, 0, n, grad, logits)
        torch.cuda.synchronize()
        gh = grad.cpu().numpy() / R
        assert np.isfinite(gh).all()
        m = 0.9 * m + 0.1 * gh                                         # Adam, ascent on the expected return
        v = 0.999 * v + 0.001 * gh * gh
        theta = (theta + lr * (m / (1 - 0.9 ** (it + 1))) / (np.sqrt(v / (1 - 0.999 ** (it + 1))) + 1e-8)).astype(np.float32)
        history.append(float(runtime.mean()))
        wt.close()
    g.close()
    print(f"[training] mean run time: first 3 iterations {np.mean(history[:3]):.2f}, last 3 {np.mean(history[-3:]):.2f}, "
          f"serial sum {n}", flush=True)
    assert np.mean(history[:3]) > 1.5 * n            # a random policy scatters the graph over the devices
    assert np.mean(history[-3:]) <= 1.05 * n         # the trained one keeps it together
