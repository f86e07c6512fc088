"""GPU parity of the on-device MDP transition and episode loop (Section 2.1) against the
float64 oracle (oracle/episode.py + the forward oracle), through the C ABI.

The sampled action is an integer decided by floating point: the kernel decides in fp32 on its
own logits, the oracle in float64 on the same logits; they may differ only where the uniform
number lies within MARGIN of a boundary of the cumulative distribution, and then only by
picking the neighbouring device.  Everything the transition writes is compared bit for bit
given the action; each step's logits are compared with the oracle's forward pass on the same
state (the oracle replays the device's actions)."""
import numpy as np
import pytest

import oracle
from oracle import episode as ep
from workloads import make_workload, make_episode

from gpu_common import assert_logits_close

pytestmark = pytest.mark.gpu
MARGIN = 1e-5


def check_action(logits_row, u, a_gpu, what):
    a_ref = ep.sample_action(logits_row.astype(np.float64), float(u))
    if a_gpu == a_ref:
        return
    assert ep.decision_margin(logits_row.astype(np.float64), float(u)) < MARGIN and abs(a_gpu - a_ref) == 1, \
        f"{what}: action {a_gpu}, oracle {a_ref}, u {u}, logits {logits_row}"


def test_single_transition_on_synthetic_logits():
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    w = make_workload("layered200", B=40)
    D = w.D
    rng = np.random.default_rng(77)
    order, _, _ = make_episode(w, 1)
    t = 3
    logits = (rng.normal(size=(w.B, D)) * 2).astype(np.float32)
    logits[0] = 0.0                                   # uniform
    logits[1] = [0.0, 60.0, 0.0, -5.0]                # saturated
    logits[2] = [1e6, 1e6 - 1.0, 1e6 - 2.0, -1e6]     # large scale, as the raw features give
    u = rng.random(w.B, dtype=np.float32)
    u[0], u[3], u[4] = 0.25, 0.0, np.float32(1.0 - 2.0 ** -24)
    placement = rng.integers(0, D, size=w.n_tot).astype(np.int32)
    feats = np.array(w.node_feats, dtype=np.float32)
    feats[:, 2] = 0.0
    cur = np.array([order[w.node_off[b] + t] for b in range(w.B)], dtype=np.int32)
    cur[5] = -1                                       # an episode that is over
    cur[6] = int(w.n_nodes[6])                        # outside the graph
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    t_l, t_u, t_o = (torch.from_numpy(x).to(dev) for x in (logits, u, order))
    t_f, t_p, t_c = (torch.from_numpy(x.copy()).to(dev) for x in (feats, placement, cur))
    act = torch.full((w.B,), 99, dtype=torch.int32, device=dev)
    logp = torch.full((w.B,), float("nan"), dtype=torch.float32, device=dev)
    pl.episode_step(g, D, t_l, t_u, t_o, t, t_f, t_p, t_c, act, logp)
    torch.cuda.synchronize()
    act, logp = act.cpu().numpy(), logp.cpu().numpy()
    new_f, new_p, new_c = t_f.cpu().numpy(), t_p.cpu().numpy(), t_c.cpu().numpy()
    exp_p, exp_f = placement.copy(), feats.copy()
    for b in range(w.B):
        n0, n_b = int(w.node_off[b]), int(w.n_nodes[b])
        if b in (5, 6):
            assert act[b] == -1 and logp[b] == 0.0 and new_c[b] == -1
            continue
        check_action(logits[b], u[b], int(act[b]), f"graph {b}")
        assert abs(logp[b] - ep.log_prob(logits[b].astype(np.float64), int(act[b]))) <= 1e-5 * max(1.0, abs(logp[b]))
        vis = exp_f[n0:n0 + n_b, 2].astype(np.float64)
        nxt = ep.transition(exp_p[n0:n0 + n_b], vis, order[n0:n0 + n_b], t, int(cur[b]), int(act[b]))
        exp_f[n0:n0 + n_b, 2] = vis
        assert new_c[b] == nxt
    np.testing.assert_array_equal(new_p, exp_p)
    np.testing.assert_array_equal(new_f, exp_f)
    assert act[0] == 1 and act[1] == 1 and act[3] == ep.sample_action(logits[3].astype(np.float64), 0.0)
    g.close()


def replay(w, b, order, uniforms, placement0, actions):
    """The oracle's episode of graph b with the device's actions forced."""
    n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
    e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
    blob = oracle.weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    base = np.array(w.node_feats[n0:n1], dtype=np.float64)

    def fwd(placement, visited, cur):
        feats = base.copy()
        feats[:, 2] = visited
        return oracle.forward_graph(n1 - n0, w.edge_src[e0:e1], w.edge_dst[e0:e1], feats, placement, cur,
                                    blob, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device)["logits"]

    return ep.run_episode(fwd, n1 - n0, placement0[n0:n1], order[n0:n1], uniforms[:, b], actions=actions)


def run_device_episode(w, n_steps, order, uniforms, placement0):
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    feats = np.array(w.node_feats, dtype=np.float32)
    feats[:, 2] = 0.0
    cur = np.array([order[w.node_off[b]] for b in range(w.B)], dtype=np.int32)
    t_f, t_p, t_c, t_o, t_u = (torch.from_numpy(np.ascontiguousarray(x)).to(dev)
                               for x in (feats, placement0, cur, order, uniforms))
    logits = torch.full((n_steps, w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    act = torch.full((n_steps, w.B), 99, dtype=torch.int32, device=dev)
    logp = torch.full((n_steps, w.B), float("nan"), dtype=torch.float32, device=dev)
    pl.episode_run(g, wt, t_f, t_p, t_c, t_o, t_u, 0, n_steps, logits, True, act, logp)
    torch.cuda.synchronize()
    out = dict(logits=logits.cpu().numpy(), actions=act.cpu().numpy(), logp=logp.cpu().numpy(),
               placement=t_p.cpu().numpy(), visited=t_f.cpu().numpy()[:, 2], cur=t_c.cpu().numpy())
    g.close()
    wt.close()
    return out


def check_against_replay(w, b, n_steps, order, uniforms, placement0, dev_out, complete):
    n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
    T = min(n_steps, n1 - n0)
    r = replay(w, b, order, uniforms[:T], placement0, dev_out["actions"][:T, b])
    assert_logits_close(dev_out["logits"][:T, b], r["logits"], f"{w.name} graph {b}: logits of every step", 0.1)
    for t in range(T):
        check_action(dev_out["logits"][t, b], uniforms[t, b], int(dev_out["actions"][t, b]), f"graph {b} step {t}")
        lp = ep.log_prob(dev_out["logits"][t, b].astype(np.float64), int(dev_out["actions"][t, b]))
        assert abs(dev_out["logp"][t, b] - lp) <= 1e-5 * max(1.0, abs(lp)), (b, t)
    np.testing.assert_array_equal(dev_out["placement"][n0:n1], r["placement"])
    np.testing.assert_array_equal(dev_out["visited"][n0:n1], r["visited"].astype(np.float32))
    assert dev_out["cur"][b] == r["cur"]
    if complete:                                      # Section 2.1: |V| steps visit every node once
        assert r["cur"] == -1 and r["visited"].sum() == n1 - n0
        assert (dev_out["actions"][T:, b] == -1).all() and (dev_out["logp"][T:, b] == 0).all()


@pytest.mark.parametrize("name,B", [("random32", 1), ("layered200", 6)])
def test_whole_episode_matches_oracle_replay(name, B):
    w = make_workload(name, B=B)
    n_steps = int(w.n_nodes.max()) + 2                # two steps past the end: nothing may change
    order, uniforms, placement0 = make_episode(w, n_steps)
    out = run_device_episode(w, n_steps, order, uniforms, placement0)
    for b in range(w.B):
        check_against_replay(w, b, n_steps, order, uniforms, placement0, out, complete=True)


def test_episode_segment_at_full_size():
    # the batch and launch configuration that the benchmark times; two graphs are replayed
    w = make_workload("nasnet")
    n_steps = 6
    order, uniforms, placement0 = make_episode(w, n_steps)
    out = run_device_episode(w, n_steps, order, uniforms, placement0)
    assert np.isfinite(out["logits"]).all()
    assert ((out["actions"] >= 0) & (out["actions"] < w.D)).all()
    for b in (0, w.B - 1):
        check_against_replay(w, b, n_steps, order, uniforms, placement0, out, complete=False)
    # every graph: exactly n_steps nodes visited, those of its order, placed where the actions say
    for b in range(w.B):
        n0 = int(w.node_off[b])
        first = order[n0:n0 + n_steps] + n0
        assert out["visited"][n0:int(w.node_off[b + 1])].sum() == n_steps
        np.testing.assert_array_equal(out["placement"][first], out["actions"][:, b])
        assert out["cur"][b] == order[n0 + n_steps]


def test_episode_loop_replays_from_a_hip_graph():
    """Sixteen steps of forward pass + transition captured once (with the reset of the state)
    and replayed three times, with eager work in between: the actions equal the eager run's."""
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    w = make_workload("layered200", B=12)
    T = 16
    order, uniforms, placement0 = make_episode(w, T)
    eager = run_device_episode(w, T, order, uniforms, placement0)
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    f0 = np.array(w.node_feats, dtype=np.float32)
    f0[:, 2] = 0.0
    cur0 = np.array([order[w.node_off[b]] for b in range(w.B)], dtype=np.int32)
    tf0, tp0, tc0, to, tu = (torch.from_numpy(np.ascontiguousarray(x)).to(dev)
                             for x in (f0, placement0, cur0, order, uniforms))
    tf, tp, tc = tf0.clone(), tp0.clone(), tc0.clone()
    logits = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
    act = torch.empty((T, w.B), dtype=torch.int32, device=dev)
    pl.embed_forward(g, tf, tp, tc, wt, logits)                     # first call allocates
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        tf.copy_(tf0); tp.copy_(tp0); tc.copy_(tc0)
        pl.episode_run(g, wt, tf, tp, tc, to, tu, 0, T, logits, False, act, None, stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for _ in range(3):
        act.fill_(77)
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(act.cpu().numpy(), eager["actions"])
        np.testing.assert_array_equal(tp.cpu().numpy(), eager["placement"])
        pl.embed_forward(g, tf0, tp0, tc0, wt, logits)              # eager work between the replays
        torch.cuda.synchronize()
    del graph
    g.close()
    wt.close()


def test_ragged_batch_graphs_finish_at_different_steps():
    """Graphs of 3, 11 and 26 nodes in one batch: each episode ends after its own |V| steps and
    is left untouched afterwards, while the others go on."""
    from workloads import tiny_random_dag, weight_count
    from workloads.synthetic import Workload
    rng = np.random.default_rng(21)
    sizes, D, H = [3, 11, 26], 3, 32
    n_nodes, n_edges, srcs, dsts, feats = [], [], [], [], []
    for n in sizes:
        s, d = tiny_random_dag(rng, n, 0.3)
        n_nodes.append(n); n_edges.append(len(s)); srcs.append(s); dsts.append(d)
        feats.append(np.stack([rng.lognormal(0, 1, n), rng.lognormal(2, 1, n), np.zeros(n)], axis=1))
    w = Workload(name="ragged", B=len(sizes), D=D, H=H, n_layers=2, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 n_nodes=np.array(n_nodes, np.int32), n_edges=np.array(n_edges, np.int32),
                 edge_src=np.concatenate(srcs).astype(np.int32), edge_dst=np.concatenate(dsts).astype(np.int32),
                 node_feats=np.concatenate(feats).astype(np.float32), placement=np.zeros(sum(sizes), np.int32),
                 cur_node=np.zeros(len(sizes), np.int32),
                 weights=rng.normal(0, 0.1, weight_count(D, H, 2, True)).astype(np.float32))
    n_steps = max(sizes) + 1
    order, uniforms, placement0 = make_episode(w, n_steps)
    out = run_device_episode(w, n_steps, order, uniforms, placement0)
    for b in range(w.B):
        check_against_replay(w, b, n_steps, order, uniforms, placement0, out, complete=True)
