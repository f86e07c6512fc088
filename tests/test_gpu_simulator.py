"""GPU parity of the placement run-time simulator against its oracle (oracle/simulator.py),
through the C ABI.  Timestamps are float32 with the same roundings on both sides and events
are ordered by (timestamp, creation number), so run times and event counts must be equal bit
for bit."""
import numpy as np
import pytest

from oracle import simulator as sim
from workloads import make_workload, tiny_random_dag
from workloads.synthetic import Workload

pytestmark = pytest.mark.gpu


def run_device(w, placement, inv_bw):
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    out = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    ev = torch.full((w.B,), -7, dtype=torch.int32, device=dev)
    pl.simulate_runtime(g, w.D, torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev),
                        torch.from_numpy(np.ascontiguousarray(placement, dtype=np.int32)).to(dev), inv_bw, out, ev)
    torch.cuda.synchronize()
    g.close()
    return out.cpu().numpy(), ev.cpu().numpy()


def oracle_graph(w, b, placement, inv_bw):
    n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
    e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
    return sim.simulate(n1 - n0, w.edge_src[e0:e1], w.edge_dst[e0:e1], w.node_feats[n0:n1, 0],
                        w.node_feats[n0:n1, 1], placement[n0:n1], w.D, inv_bw)


@pytest.mark.parametrize("name,B,inv_bw", [("random32", 1, 1e-4), ("layered200", 8, 1e-4), ("inception", 4, 3e-5),
                                           ("nmt", 3, 1e-4), ("nasnet", 3, 5e-5), ("layered200", 5, 0.0)])
def test_run_times_and_event_counts_bit_exact(name, B, inv_bw):
    w = make_workload(name, B=B)
    rng = np.random.default_rng(17)
    for trial in range(2):
        placement = w.placement if trial == 0 else rng.integers(0, w.D, w.n_tot).astype(np.int32)
        got_r, got_e = run_device(w, placement, inv_bw)
        for b in range(w.B):
            r, e = oracle_graph(w, b, placement, np.float32(inv_bw))
            assert got_e[b] == e, (name, b, got_e[b], e)
            assert got_r[b] == r, (name, b, got_r[b], r)


def test_all_on_one_device_and_bad_device_ids():
    w = make_workload("layered200", B=4)
    placement = np.zeros(w.n_tot, dtype=np.int32)
    placement[w.node_off[2] + 5] = w.D            # outside [0, D): that graph only
    got_r, got_e = run_device(w, placement, 1e-4)
    for b in range(w.B):
        n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
        if b == 2:
            assert np.isnan(got_r[b]) and got_e[b] == -1
        else:
            assert got_e[b] == n1 - n0           # no transfers
            assert abs(got_r[b] - w.node_feats[n0:n1, 0].astype(np.float64).sum()) <= 1e-4 * got_r[b]


@pytest.mark.parametrize("D", [1, 5, 16])
def test_random_dags_with_ties_and_wide_fan_out(D):
    # integer costs and sizes: many events share a timestamp, so the tie rules decide the order
    rng = np.random.default_rng(3)
    sizes = [1, 2, 30, 64, 100, 7]
    n_nodes, n_edges, srcs, dsts, feats = [], [], [], [], []
    for n in sizes:
        s, d = tiny_random_dag(rng, n, 0.3)
        n_nodes.append(n); n_edges.append(len(s)); srcs.append(s); dsts.append(d)
        feats.append(np.stack([rng.integers(1, 4, n), rng.integers(0, 3, n), np.zeros(n)], axis=1))
    w = Workload(name="custom", B=len(sizes), D=D, H=8, n_layers=1, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 n_nodes=np.array(n_nodes, np.int32), n_edges=np.array(n_edges, np.int32),
                 edge_src=np.concatenate(srcs).astype(np.int32), edge_dst=np.concatenate(dsts).astype(np.int32),
                 node_feats=np.concatenate(feats).astype(np.float32),
                 placement=rng.integers(0, D, sum(sizes)).astype(np.int32),
                 cur_node=np.zeros(len(sizes), np.int32), weights=np.zeros(1, np.float32))
    got_r, got_e = run_device(w, w.placement, 1.0)
    for b in range(w.B):
        r, e = oracle_graph(w, b, w.placement, np.float32(1.0))
        assert (got_r[b], got_e[b]) == (r, e), (b, got_r[b], r, got_e[b], e)


def test_full_batch_sampled():
    # the benchmark's batch; three graphs are simulated by the oracle
    w = make_workload("nasnet")
    got_r, got_e = run_device(w, w.placement, 5e-5)
    assert np.isfinite(got_r).all() and (got_e >= w.n_nodes).all()
    for b in (0, 100, w.B - 1):
        r, e = oracle_graph(w, b, w.placement, np.float32(5e-5))
        assert (got_r[b], got_e[b]) == (r, e)


# ---------------------------------------------------------------- peak memory and R(p)
def run_device_reward(w, placement, inv_bw, M, c, handles=None):
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    g = handles or pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    rew = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    rt = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    peak = torch.full((w.B, w.D), -1.0, dtype=torch.float32, device=dev)
    ev = torch.full((w.B,), -7, dtype=torch.int32, device=dev)
    pl.simulate_reward(g, w.D, torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev),
                       torch.from_numpy(np.ascontiguousarray(placement, dtype=np.int32)).to(dev), inv_bw, M, c,
                       rew, rt, peak, ev)
    torch.cuda.synchronize()
    if handles is None:
        g.close()
    return rew.cpu().numpy(), rt.cpu().numpy(), peak.cpu().numpy(), ev.cpu().numpy()


def oracle_reward(w, b, placement, inv_bw, M, c):
    n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
    e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
    n, src, dst = n1 - n0, w.edge_src[e0:e1], w.edge_dst[e0:e1]
    size = w.node_feats[n0:n1, 1]
    r, st, en, arr = sim.timeline(n, src, dst, w.node_feats[n0:n1, 0], size, placement[n0:n1], w.D, np.float32(inv_bw))
    peak = sim.peak_memory(n, src, dst, size, placement[n0:n1], w.D, st, en, arr)
    return r, peak, sim.penalised_runtime(r, peak.max(), M, c)


@pytest.mark.parametrize("name,B,inv_bw", [("random32", 1, 1e-4), ("layered200", 8, 1e-4), ("inception", 3, 3e-5),
                                           ("nmt", 2, 1e-4), ("nasnet", 2, 5e-5)])
def test_peak_memory_and_penalised_run_time(name, B, inv_bw):
    """Run time bit for bit; peaks (float64 sums rounded once to fp32) and R(p) to 1e-6 relative.  The
    limit M is set between the smallest and the largest peak of the batch, so both branches of R(p)
    occur."""
    w = make_workload(name, B=B)
    rng = np.random.default_rng(23)
    for trial in range(2):
        placement = w.placement if trial == 0 else rng.integers(0, w.D, w.n_tot).astype(np.int32)
        refs = [oracle_reward(w, b, placement, inv_bw, 0.0, 0.0) for b in range(w.B)]
        peaks = np.array([p.max() for _, p, _ in refs])
        M = float(np.float32(0.5 * (peaks.min() + peaks.max())))
        c = 2.0 * float(max(r for r, _, _ in refs)) / float(peaks.max())    # a penalty of the run time's size
        rew, rt, peak, ev = run_device_reward(w, placement, inv_bw, M, c)
        above = 0
        for b in range(w.B):
            r, p, _ = refs[b]
            assert rt[b] == r, (name, b)
            np.testing.assert_allclose(peak[b], p, rtol=1e-6, atol=0, err_msg=f"{name} graph {b}")
            want = sim.penalised_runtime(r, p.max(), M, np.float32(c))
            assert abs(rew[b] - want) <= 2e-6 * abs(want), (name, b, rew[b], want)
            above += p.max() > M
        if w.B > 1:
            assert 0 < above < w.B or peaks.min() == peaks.max()


def test_reward_edge_cases():
    """One device (nothing ever crosses), an edgeless graph, a bad device id, and the plain run time
    when the limit is never reached."""
    rng = np.random.default_rng(4)
    n = 30
    src, dst = tiny_random_dag(rng, n, 0.2)
    feats = np.stack([rng.integers(1, 6, n), rng.integers(1, 50, n), np.zeros(n)], axis=1).astype(np.float32)
    for D, edges in ((1, (src, dst)), (3, (np.zeros(0, np.int32), np.zeros(0, np.int32))), (4, (src, dst))):
        placement = rng.integers(0, D, n).astype(np.int32)
        w = Workload(name="t", B=1, D=D, H=8, n_layers=1, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                     n_nodes=np.array([n], np.int32), n_edges=np.array([len(edges[0])], np.int32),
                     edge_src=edges[0], edge_dst=edges[1], node_feats=feats, placement=placement,
                     cur_node=np.zeros(1, np.int32), weights=np.zeros(1, np.float32))
        r, p, _ = oracle_reward(w, 0, placement, 0.25, 0.0, 0.0)
        rew, rt, peak, ev = run_device_reward(w, placement, 0.25, 1e9, 2.0)
        assert rt[0] == r and rew[0] == r                      # below the limit: R(p) = r
        np.testing.assert_allclose(peak[0], p, rtol=1e-6)
        rew, _, _, _ = run_device_reward(w, placement, 0.25, 0.0, 2.0)
        assert abs(rew[0] - (float(r) + 2.0 * p.max())) <= 2e-6 * (float(r) + 2.0 * p.max())
    bad = placement.copy()
    bad[3] = 9
    rew, rt, peak, ev = run_device_reward(w, bad, 0.25, 1.0, 2.0)
    assert np.isnan(rew[0]) and np.isnan(rt[0]) and np.isnan(peak[0]).all() and ev[0] == -1


def test_full_batch_reward_sampled_graphs():
    w = make_workload("nasnet")
    rng = np.random.default_rng(31)
    placement = rng.integers(0, w.D, w.n_tot).astype(np.int32)
    rew, rt, peak, ev = run_device_reward(w, placement, 5e-5, 0.0, 1e-6)
    for b in (0, 77, 255):
        r, p, want = oracle_reward(w, b, placement, 5e-5, 0.0, np.float32(1e-6))
        assert rt[b] == r
        np.testing.assert_allclose(peak[b], p, rtol=1e-6)
        assert abs(rew[b] - want) <= 2e-6 * abs(want)


# ---------------------------------------------------------------- one transfer per child
def _device_both(w, placement, inv_bw, per_child, M=1e30, c=2.0):
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    f = torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev)
    p = torch.from_numpy(np.ascontiguousarray(placement, dtype=np.int32)).to(dev)
    rt = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    ev = torch.full((w.B,), -7, dtype=torch.int32, device=dev)
    pl.simulate_runtime(g, w.D, f, p, inv_bw, rt, ev, per_child_transfers=per_child)
    rew = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    rt2 = torch.full((w.B,), -1.0, dtype=torch.float32, device=dev)
    peak = torch.full((w.B, w.D), -1.0, dtype=torch.float32, device=dev)
    ev2 = torch.full((w.B,), -7, dtype=torch.int32, device=dev)
    pl.simulate_reward(g, w.D, f, p, inv_bw, M, c, rew, rt2, peak, ev2, per_child_transfers=per_child)
    torch.cuda.synchronize()
    g.close()
    np.testing.assert_array_equal(rt.cpu().numpy(), rt2.cpu().numpy())
    np.testing.assert_array_equal(ev.cpu().numpy(), ev2.cpu().numpy())
    return rt.cpu().numpy(), ev.cpu().numpy(), peak.cpu().numpy(), rew.cpu().numpy()


def _oracle_both(w, b, placement, inv_bw, per_child):
    n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
    e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
    n, src, dst = n1 - n0, w.edge_src[e0:e1], w.edge_dst[e0:e1]
    cost, size = w.node_feats[n0:n1, 0], w.node_feats[n0:n1, 1]
    r, e = sim.simulate(n, src, dst, cost, size, placement[n0:n1], w.D, np.float32(inv_bw), per_child=bool(per_child))
    r2, st, en, arr = sim.timeline(n, src, dst, cost, size, placement[n0:n1], w.D, np.float32(inv_bw), per_child=bool(per_child))
    assert r2 == r
    return r, e, sim.peak_memory(n, src, dst, size, placement[n0:n1], w.D, st, en, arr)


def test_two_children_on_one_remote_device_on_the_device():
    """The hand-computed example of the oracle's pin (tests/test_oracle_simulator.py): r = 5 with one
    transfer per destination device, r = 6 with one per child; peaks 2048 / 2560."""
    w = Workload(name="t", B=1, D=2, H=8, n_layers=1, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 n_nodes=np.array([3], np.int32), n_edges=np.array([2], np.int32), edge_src=np.array([0, 0], np.int32),
                 edge_dst=np.array([1, 2], np.int32),
                 node_feats=np.array([[1, 2048, 0], [1, 512, 0], [1, 256, 0]], np.float32),
                 placement=np.array([0, 1, 1], np.int32), cur_node=np.zeros(1, np.int32), weights=np.zeros(1, np.float32))
    rt, ev, peak, _ = _device_both(w, w.placement, 1.0 / 1024.0, 0)
    assert (rt[0], ev[0]) == (5.0, 4) and list(peak[0]) == [2048.0, 2560.0]
    rt, ev, peak, _ = _device_both(w, w.placement, 1.0 / 1024.0, 1)
    assert (rt[0], ev[0]) == (6.0, 5) and list(peak[0]) == [2048.0, 2560.0]


@pytest.mark.parametrize("name,B,inv_bw", [("random32", 1, 1e-4), ("layered200", 8, 1e-4), ("inception", 3, 3e-5),
                                           ("nmt", 2, 1e-4), ("nasnet", 2, 5e-5)])
def test_per_child_transfers_bit_exact(name, B, inv_bw):
    """The printed op-done / transfer-done handlers (one transfer per child on another device): run
    times and event counts bit for bit, peaks to 1e-6 relative, on every workload; the run differs
    from the default wherever an operation has two children on one remote device."""
    w = make_workload(name, B=B)
    rng = np.random.default_rng(29)
    differs = 0
    for trial in range(2):
        placement = w.placement if trial == 0 else rng.integers(0, w.D, w.n_tot).astype(np.int32)
        rt, ev, peak, _ = _device_both(w, placement, inv_bw, 1)
        rt0, ev0, _, _ = _device_both(w, placement, inv_bw, 0)
        for b in range(w.B):
            r, e, p = _oracle_both(w, b, placement, inv_bw, 1)
            assert (rt[b], ev[b]) == (r, e), (name, b, rt[b], r, ev[b], e)
            np.testing.assert_allclose(peak[b], p, rtol=1e-6, atol=0, err_msg=f"{name} graph {b}")
            n0, n1 = int(w.node_off[b]), int(w.node_off[b + 1])
            e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
            crossing = int((placement[n0:n1][w.edge_src[e0:e1]] != placement[n0:n1][w.edge_dst[e0:e1]]).sum())
            assert ev[b] == (n1 - n0) + crossing
            differs += ev[b] != ev0[b]
    assert differs > 0 or name == "random32"


def test_per_child_transfers_with_ties_and_at_full_size():
    rng = np.random.default_rng(8)
    sizes = [1, 2, 30, 64, 100, 7]
    n_nodes, n_edges, srcs, dsts, feats = [], [], [], [], []
    for n in sizes:
        s, d = tiny_random_dag(rng, n, 0.3)
        n_nodes.append(n); n_edges.append(len(s)); srcs.append(s); dsts.append(d)
        feats.append(np.stack([rng.integers(1, 4, n), rng.integers(0, 3, n), np.zeros(n)], axis=1))
    w = Workload(name="custom", B=len(sizes), D=3, H=8, n_layers=1, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 n_nodes=np.array(n_nodes, np.int32), n_edges=np.array(n_edges, np.int32),
                 edge_src=np.concatenate(srcs).astype(np.int32), edge_dst=np.concatenate(dsts).astype(np.int32),
                 node_feats=np.concatenate(feats).astype(np.float32),
                 placement=rng.integers(0, 3, sum(sizes)).astype(np.int32),
                 cur_node=np.zeros(len(sizes), np.int32), weights=np.zeros(1, np.float32))
    rt, ev, peak, _ = _device_both(w, w.placement, 1.0, 1)
    for b in range(w.B):
        r, e, p = _oracle_both(w, b, w.placement, 1.0, 1)
        assert (rt[b], ev[b]) == (r, e), b
        np.testing.assert_allclose(peak[b], p, rtol=1e-6, atol=0)
    w = make_workload("nasnet")
    rt, ev, peak, _ = _device_both(w, w.placement, 5e-5, 1)
    for b in (0, 131, w.B - 1):
        r, e, p = _oracle_both(w, b, w.placement, 5e-5, 1)
        assert (rt[b], ev[b]) == (r, e), b
        np.testing.assert_allclose(peak[b], p, rtol=1e-6, atol=0)
