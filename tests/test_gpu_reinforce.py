"""GPU parity of the REINFORCE accumulation (appendix "REINFORCE Algorithm", Eq. 1):
pl_reinforce_coeff against the float64 oracle, and one whole policy-gradient estimate - rollouts
on the device, simulated run times as rewards, return-minus-baseline weights, replay with
gradients - against the composition of the oracles, through the C ABI."""
import numpy as np
import pytest

import oracle
from oracle import episode as oe, gradient as og, reinforce as orf, simulator as osim
from gpu_common import custom_workload
from test_gpu_gradient import assert_grad_close
from workloads import make_workload, make_episode
from workloads.synthetic import Workload

pytestmark = pytest.mark.gpu


def test_weights_of_the_sum_against_the_oracle():
    import torch
    import paper_1906_08879_amd as pl
    rng = np.random.default_rng(3)
    for T, B, n_groups in ((37, 23, 5), (1, 1, 1), (300, 64, 64), (12, 7, 0)):
        r = rng.normal(0, 1, (T, B)).astype(np.float32)
        group = rng.integers(0, max(n_groups, 1), B).astype(np.int32)
        if B > 3:
            group[2] = n_groups + 3                              # outside the range: plain return
        dev = torch.device("cuda:0")
        coeff = torch.full((T, B), float("nan"), dtype=torch.float32, device=dev)
        base = torch.full((T, max(n_groups, 1)), float("nan"), dtype=torch.float32, device=dev)
        pl.reinforce_coeff(torch.from_numpy(r).to(dev), torch.from_numpy(group).to(dev), n_groups, coeff,
                           base if n_groups else None)
        torch.cuda.synchronize()
        ref_c, ref_b = orf.advantages(r, group, n_groups)
        scale = np.abs(orf.returns_to_go(r)).max()
        assert np.abs(coeff.cpu().numpy() - ref_c).max() <= 2e-6 * scale, (T, B)
        if n_groups:
            assert np.abs(base.cpu().numpy()[:, :n_groups] - ref_b).max() <= 2e-6 * scale, (T, B)


def _rollout_batch(w, rollouts):
    """`rollouts` copies of each graph of a workload, side by side in one batch."""
    n_graphs, name = w.B, w.name
    parts = dict(n_nodes=[], n_edges=[], src=[], dst=[], feats=[], place=[], cur=[], group=[])
    for b in range(n_graphs):
        n, src, dst, feats, placement, cur = w.graph(b)
        for _ in range(rollouts):
            parts["n_nodes"].append(n); parts["n_edges"].append(len(src)); parts["src"].append(src)
            parts["dst"].append(dst); parts["feats"].append(feats); parts["place"].append(placement)
            parts["cur"].append(cur); parts["group"].append(b)
    wb = Workload(name=name + "-rollouts", B=n_graphs * rollouts, D=w.D, H=w.H, n_layers=w.n_layers,
                  k_sweeps=w.k_sweeps, group_by_device=w.group_by_device, weight_dtype=w.weight_dtype,
                  n_nodes=np.array(parts["n_nodes"], np.int32), n_edges=np.array(parts["n_edges"], np.int32),
                  edge_src=np.concatenate(parts["src"]).astype(np.int32),
                  edge_dst=np.concatenate(parts["dst"]).astype(np.int32),
                  node_feats=np.concatenate(parts["feats"]).astype(np.float32),
                  placement=np.concatenate(parts["place"]).astype(np.int32),
                  cur_node=np.array(parts["cur"], np.int32), weights=w.weights)
    return wb, np.array(parts["group"], np.int32)


@pytest.mark.parametrize("name,rollouts", [("generic", 3), ("ragged", 2)])
def test_one_policy_gradient_estimate_end_to_end(name, rollouts):
    """Rollouts of the same graphs under one policy (different random numbers), intermediate
    rewards = decrease of the simulated run time at every step (Appendix A.7 "Intermediate
    Rewards"), baseline = mean over the rollouts of the graph, gradient by replay, with an entropy
    term per decision (Appendix A.7 "Entropy")."""
    import torch
    import paper_1906_08879_amd as pl
    if name == "ragged":     # graphs of different length on the matrix-core path (H = 32, fp32 weights)
        base_w = custom_workload(np.random.default_rng(8), [40, 25], 4, 32, w_scale=0.15)
    else:                    # generic kernels (H = 8), three devices
        base_w = custom_workload(np.random.default_rng(9), [20, 14], 3, 8, w_scale=0.1)
    n_graphs = base_w.B
    w, group = _rollout_batch(base_w, rollouts)
    T = int(w.n_nodes.max())
    order, uniforms, placement0 = make_episode(w, T, seed=11)
    for b in range(w.B):                                            # rollouts of a graph share its visiting order
        first = int(np.flatnonzero(group == group[b])[0])
        n = int(w.n_nodes[b])
        order[w.node_off[b]:w.node_off[b] + n] = order[w.node_off[first]:w.node_off[first] + n]
    dev = torch.device("cuda:0")
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    f0 = np.array(w.node_feats, dtype=np.float32, copy=True)
    f0[:, 2] = 0.0
    cur0 = np.array([order[w.node_off[b]] for b in range(w.B)], dtype=np.int32)
    inv_bw = 1e-4
    print(f"[reinforce] {name}: rollout of {T} steps", flush=True)
    d_f, d_p, d_c = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (f0, placement0, cur0))
    d_o, d_u = torch.from_numpy(order).to(dev), torch.from_numpy(uniforms).to(dev)
    logits = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
    actions = torch.empty((T, w.B), dtype=torch.int32, device=dev)
    logp_roll = torch.empty((T, w.B), dtype=torch.float32, device=dev)
    runtime = torch.empty((T + 1, w.B), dtype=torch.float32, device=dev)
    pl.simulate_runtime(g, w.D, d_f, d_p, inv_bw, runtime[0])
    for t in range(T):
        pl.episode_run(g, wt, d_f, d_p, d_c, d_o, d_u[t:t + 1], t, 1, logits, False, actions[t:t + 1], logp_roll[t:t + 1])
        pl.simulate_runtime(g, w.D, d_f, d_p, inv_bw, runtime[t + 1])
    rewards = (runtime[:-1] - runtime[1:]).contiguous()             # improvement of the run time
    coeff = torch.empty((T, w.B), dtype=torch.float32, device=dev)
    base = torch.empty((T, n_graphs), dtype=torch.float32, device=dev)
    pl.reinforce_coeff(rewards, torch.from_numpy(group).to(dev), n_graphs, coeff, base)
    # replay from the initial state
    d_f, d_p, d_c = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (f0, placement0, cur0))
    n_par = pl.weights_count(w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    grad = torch.full((n_par,), float("nan"), dtype=torch.float32, device=dev)
    logp_replay = torch.empty((T, w.B), dtype=torch.float32, device=dev)
    beta = torch.from_numpy(np.random.default_rng(5).uniform(0.0, 0.5, (T, w.B)).astype(np.float32)).to(dev)
    pl.episode_gradient(g, wt, d_f, d_p, d_c, d_o, actions, coeff, 0, T, grad, logits, logp_replay, entropy_coeff=beta)
    torch.cuda.synchronize()
    act = actions.cpu().numpy()
    rt = runtime.cpu().numpy()
    live = np.arange(T)[:, None] < w.n_nodes[None, :]
    # the replay sees the states of the rollout: same log-probabilities, bit for bit
    np.testing.assert_array_equal(logp_replay.cpu().numpy()[live], logp_roll.cpu().numpy()[live])
    assert (d_c.cpu().numpy() == -1).all()

    # the oracles, with the device's actions: run times, weights, gradient
    print(f"[reinforce] {name}: oracle", flush=True)
    ref_rt = np.zeros((T + 1, w.B))
    for b in range(w.B):
        n, src, dst, feats, _, _ = w.graph(b)
        n0 = int(w.node_off[b])
        placement = np.array(placement0[n0:n0 + n], copy=True)
        cost, size = feats[:, 0], feats[:, 1]
        ref_rt[0, b] = osim.simulate(n, src, dst, cost, size, placement, w.D, inv_bw)[0]
        for t in range(T):
            if t < n:
                placement[order[n0 + t]] = act[t, b]
            ref_rt[t + 1, b] = osim.simulate(n, src, dst, cost, size, placement, w.D, inv_bw)[0]
    np.testing.assert_array_equal(rt, ref_rt.astype(np.float32))     # the simulator is bit-exact
    ref_coeff, _ = orf.advantages(ref_rt[:-1] - ref_rt[1:], group, n_graphs)
    assert np.abs(ref_coeff).max() > 0 and (act[:, 0] != act[:, 1]).any(), "degenerate case: identical rollouts"
    cscale = np.abs(ref_coeff).max()
    assert np.abs(coeff.cpu().numpy() - ref_coeff).max() <= 1e-5 * max(cscale, np.abs(ref_rt).max()), name
    ref_grad, ref_logp = orf.episode_gradient(w, order, act, ref_coeff, placement0,
                                              entropy_coeff=beta.cpu().numpy().astype(np.float64))
    assert np.abs(logp_roll.cpu().numpy() - ref_logp)[live].max() <= 2e-3
    worst = assert_grad_close(grad.cpu().numpy(), ref_grad, w, name + " REINFORCE sum")
    print(f"[reinforce] {name}: worst error / bound = {worst:.3g}", flush=True)
    g.close()
    wt.close()
