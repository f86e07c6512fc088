"""Pins for the simulator oracle (oracle/simulator.py): closed forms on small graphs, bounds
that any valid schedule obeys, and the FIFO and overlap rules the paper states."""
import numpy as np
import pytest

from oracle import simulator as sim
from workloads import make_workload, tiny_random_dag

BW = 1.0 / 1024.0     # seconds per byte in these tests is 1/1024: sizes in KiB become seconds


def run(n, edges, cost, size, place, D, inv_bw=BW, trace=None, per_child=False):
    src = [e[0] for e in edges]
    dst = [e[1] for e in edges]
    return sim.simulate(n, src, dst, cost, size, place, D, inv_bw, trace, per_child)


def test_chain_on_one_device_is_the_sum_of_costs():
    r, ev = run(4, [(0, 1), (1, 2), (2, 3)], [1, 2, 4, 8], [1024] * 4, [0, 0, 0, 0], 2)
    assert r == 15.0 and ev == 4


def test_chain_across_devices_adds_one_transfer_per_crossing():
    # 0 -(2 s)-> 1 on another device -> 2 back: 1 + 2 + 2 + 3 + 4
    r, ev = run(3, [(0, 1), (1, 2)], [1, 2, 4], [2048, 3072, 0], [0, 1, 0], 2)
    assert r == 1 + 2 + 2 + 3 + 4 and ev == 5


def test_independent_ops_run_in_parallel_on_two_devices_and_serially_on_one():
    assert run(2, [], [3, 5], [0, 0], [0, 1], 2)[0] == 5.0
    assert run(2, [], [3, 5], [0, 0], [0, 0], 2)[0] == 8.0


def test_fork_join_with_overlapping_transfer():
    # 0 -> {1 (same device), 2 (other device)} -> 3 on device 0.
    # t=1: 0 done, 1 starts on dev 0 (till 3), tensor 0 leaves (1 s) -> 2 runs 2..6 on dev 1,
    # tensor 2 travels 6..7, 3 runs 7..8: communication overlapped op 1's compute.
    trace = []
    r, _ = run(4, [(0, 1), (0, 2), (1, 3), (2, 3)], [1, 2, 4, 1], [1024, 1024, 1024, 0], [0, 0, 1, 0], 2,
               trace=trace)
    assert r == 8.0
    assert ("tr", 0, 1, 2.0) in trace and ("op", 2, 1, 6.0) in trace and ("tr", 2, 0, 7.0) in trace


def test_one_transfer_per_destination_device_and_bus_is_fifo():
    # 0 has three children on device 1: its output crosses once.  The bus of device 0 carries
    # 0's tensor (4 s) before 1's (1 s) although 1's consumer would be ready first.
    trace = []
    r, ev = run(6, [(0, 2), (0, 3), (0, 4), (1, 5)], [1, 1, 1, 1, 1, 1], [4096, 1024, 0, 0, 0, 0],
                [0, 0, 1, 1, 1, 1], 2, trace=trace)
    trs = [t for t in trace if t[0] == "tr"]
    assert trs == [("tr", 0, 1, 5.0), ("tr", 1, 1, 6.0)]
    assert ev == 6 + 2
    # device 1 runs 2, 3, 4 (ready at 5, ascending ids), then 5 (ready at 6): 5..9
    assert r == 9.0


def test_two_children_on_one_remote_device_one_transfer_or_two():
    """Appendix "Simulator", op-done handler read literally (one transfer per child on another
    device) against one transfer per destination device.  0 runs 0..1 on device 0; its output
    (2 s on the bus) is needed by 1 and 2 on device 1.
    Per destination: bus 1..3; 1 runs 3..4, 2 runs 4..5: r = 5, 3 + 1 events.
    Per child: bus 1..3 for child 1 and 3..5 for child 2; 1 runs 3..4, 2 runs 5..6: r = 6, 3 + 2 events."""
    g = dict(n=3, edges=[(0, 1), (0, 2)], cost=[1, 1, 1], size=[2048, 512, 256], place=[0, 1, 1], D=2)
    trace = []
    r, ev = run(**g, trace=trace)
    assert (r, ev) == (5.0, 4)
    assert [t for t in trace if t[0] == "tr"] == [("tr", 0, 1, 3.0)]
    trace = []
    r, ev = run(**g, trace=trace, per_child=True)
    assert (r, ev) == (6.0, 5)
    assert [t for t in trace if t[0] == "tr"] == [("tr", 0, 1, 3.0), ("tr", 0, 1, 5.0)]
    assert [t for t in trace if t[0] == "op"] == [("op", 0, 0, 1.0), ("op", 1, 1, 4.0), ("op", 2, 1, 6.0)]
    # peak memory with repeated crossings: 0's output stays on device 0 until its LAST transfer has
    # arrived (0..5) and is on device 1 from the FIRST arrival to the end of its last consumer
    # (3..6); 1's output lives 3..4, 2's 5..6: device 1 holds 2048 + 512 at t = 3, 2048 + 256 at t = 5
    src, dst = [0, 0], [1, 2]
    rt, start, end, arr = sim.timeline(3, src, dst, g["cost"], g["size"], g["place"], 2, BW, per_child=True)
    first, last = arr
    assert first[0, 1] == 3.0 and last[0, 1] == 5.0 and first[0, 0] == -1.0
    alloc, free = sim.tensor_lifetimes(3, src, dst, g["place"], 2, start, end, arr)
    assert (alloc[0, 0], free[0, 0]) == (0.0, 5.0) and (alloc[0, 1], free[0, 1]) == (3.0, 6.0)
    peak = sim.peak_memory(3, src, dst, g["size"], g["place"], 2, start, end, arr)
    assert list(peak) == [2048.0, 2560.0]
    # the default on the same graph: the source is released at 3, the copy lives 3..5
    rt, start, end, arr = sim.timeline(3, src, dst, g["cost"], g["size"], g["place"], 2, BW)
    alloc, free = sim.tensor_lifetimes(3, src, dst, g["place"], 2, start, end, arr)
    assert (alloc[0, 0], free[0, 0]) == (0.0, 3.0) and (alloc[0, 1], free[0, 1]) == (3.0, 5.0)


def test_per_child_transfers_on_a_mixed_fan_out():
    """0 (device 0, 1 s on the bus) feeds 1 (device 0), 2 and 3 (device 1), 4 (device 2); unit costs.
    Per destination: bus 1..2 (to 1), 2..3 (to 2); 2 runs 2..3, 3 runs 3..4, 4 runs 3..4: r = 4, 5 + 2 events.
    Per child: bus 1..2, 2..3 (both to 1), 3..4 (to 2); 2 runs 2..3, 3 runs 3..4, 4 runs 4..5: r = 5, 5 + 3 events."""
    g = dict(n=5, edges=[(0, 1), (0, 2), (0, 3), (0, 4)], cost=[1] * 5, size=[1024, 0, 0, 0, 0],
             place=[0, 0, 1, 1, 2], D=3)
    assert run(**g) == (4.0, 7)
    assert run(**g, per_child=True) == (5.0, 8)


@pytest.mark.parametrize("seed", range(6))
def test_per_child_transfers_event_count_and_agreement_without_shared_destinations(seed):
    """Per child, every edge that crosses devices is one transfer: events = n + crossing edges.
    Where no operation has two children on one remote device the two readings are the same
    simulation, event by event."""
    rng = np.random.default_rng(400 + seed)
    n, D = int(rng.integers(5, 40)), int(rng.integers(2, 5))
    src, dst = tiny_random_dag(rng, n, 0.2)
    cost, size = rng.lognormal(0, 1, n), rng.lognormal(7, 1, n)
    place = rng.integers(0, D, n)
    r, ev = sim.simulate(n, src, dst, cost, size, place, D, BW, per_child=True)
    assert ev == n + int((place[src] != place[dst]).sum())
    # a chain visits every device in turn: no shared destinations, so both readings agree exactly
    chain = [(i, i + 1) for i in range(n - 1)]
    cs, cd = [e[0] for e in chain], [e[1] for e in chain]
    t1, t2 = [], []
    a = sim.simulate(n, cs, cd, cost, size, place, D, BW, t1)
    b = sim.simulate(n, cs, cd, cost, size, place, D, BW, t2, per_child=True)
    assert a == b and t1 == t2


def test_device_queue_is_fifo_in_ready_order():
    # device 1 gets op 3 (ready at 1) before op 2 (ready at 2): FIFO by readiness, not by id
    trace = []
    run(4, [(0, 2), (1, 3)], [2, 1, 5, 5], [0, 0, 0, 0], [0, 0, 0, 0], 1, trace=trace)
    # single device: 0 (0..2), 1 (2..3), then 2 was queued at t=2, 3 at t=3
    assert [t[1] for t in trace if t[0] == "op"] == [0, 1, 2, 3]
    trace = []
    run(4, [(0, 2), (1, 3)], [2, 1, 5, 5], [0, 0, 0, 0], [0, 1, 1, 1], 2, trace=trace)
    order_on_1 = [t[1] for t in trace if t[0] == "op" and t[2] == 1]
    assert order_on_1 == [1, 3, 2]


@pytest.mark.parametrize("seed", range(6))
def test_bounds_and_single_device_sum_on_random_dags(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 40))
    src, dst = tiny_random_dag(rng, n, 0.25)
    cost = rng.lognormal(0, 1, n).astype(np.float32)
    size = rng.lognormal(3, 1, n).astype(np.float32)
    D = 3
    place = rng.integers(0, D, n)
    r, ev = sim.simulate(n, src, dst, cost, size, place, D, BW)
    # longest path of compute costs <= r <= everything serialised
    lp = np.zeros(n)
    order = np.argsort([0] * n)
    indeg = np.zeros(n, int)
    for v in dst:
        indeg[v] += 1
    ch = [[] for _ in range(n)]
    for u, v in zip(src, dst):
        ch[u].append(v)
    stack = [v for v in range(n) if indeg[v] == 0]
    for v in stack:
        lp[v] = cost[v]
    while stack:
        u = stack.pop()
        for v in ch[u]:
            lp[v] = max(lp[v], lp[u] + cost[v])
            indeg[v] -= 1
            if indeg[v] == 0:
                stack.append(v)
    n_cross = len({(u, place[v]) for u, v in zip(src, dst) if place[u] != place[v]})
    assert ev == n + n_cross
    assert r >= lp.max() * (1 - 1e-6)
    assert r <= (cost.sum() + sum(size[u] * BW for u, dv in {(u, place[v]) for u, v in zip(src, dst)
                                                               if place[u] != place[v]})) * (1 + 1e-5)
    # all on one device: no transfers, the sum of the costs in some order
    r1, ev1 = sim.simulate(n, src, dst, cost, size, np.zeros(n, int), D, BW)
    assert ev1 == n and abs(r1 - cost.astype(np.float64).sum()) <= 1e-5 * cost.sum()
    # relabelling the devices changes nothing
    perm = rng.permutation(D)
    r2, _ = sim.simulate(n, src, dst, cost, size, perm[place], D, BW)
    assert r2 == r or abs(r2 - r) <= 1e-6 * r      # wake-up order among devices may differ by ties only


def test_runs_on_a_workload_graph():
    w = make_workload("layered200", B=1)
    n, src, dst = w.graph(0)[:3]
    r, ev = sim.simulate(n, src, dst, w.node_feats[:n, 0], w.node_feats[:n, 1], w.placement[:n], w.D, 1e-9)
    assert np.isfinite(r) and r > 0 and ev >= n


# ---------------------------------------------------------------- peak memory and R(p)
def _mem(n, edges, cost, size, placement, D, inv_bw=1.0):
    src = np.array([e[0] for e in edges], dtype=np.int32)
    dst = np.array([e[1] for e in edges], dtype=np.int32)
    r, st, en, arr = sim.timeline(n, src, dst, cost, size, placement, D, inv_bw)
    return r, st, en, arr, sim.peak_memory(n, src, dst, size, placement, D, st, en, arr)


def test_peak_memory_of_a_chain_on_one_device():
    """a -> b -> c on device 0, costs 1, 2, 3, sizes 5, 7, 11.  a lives [0, 3) (until b ends), b
    [1, 6), c [3, 6): at t = 0: 5; at t = 1: 5 + 7; at t = 3: a is freed, 7 + 11."""
    r, st, en, arr, peak = _mem(3, [(0, 1), (1, 2)], [1, 2, 3], [5, 7, 11], [0, 0, 0], 2)
    np.testing.assert_array_equal(st, [0, 1, 3])
    np.testing.assert_array_equal(en, [1, 3, 6])
    assert (arr < 0).all()
    np.testing.assert_allclose(peak, [18.0, 0.0])
    # a large first tensor instead: the peak is while b runs
    _, _, _, _, peak = _mem(3, [(0, 1), (1, 2)], [1, 2, 3], [50, 7, 11], [0, 0, 0], 2)
    np.testing.assert_allclose(peak, [57.0, 0.0])


def test_peak_memory_with_a_transfer():
    """a (device 0, cost 1, size 4) -> b (device 1, cost 2, size 3), bandwidth 1: the transfer runs
    [1, 5).  Device 0 holds a from its start until the transfer has arrived; device 1 receives the
    copy at 5 and holds it, with b's output, until b ends at 7."""
    r, st, en, arr, peak = _mem(2, [(0, 1)], [1, 2], [4, 3], [0, 1], 2)
    assert r == 7 and arr[0, 1] == 5 and st[1] == 5
    np.testing.assert_allclose(peak, [4.0, 7.0])
    src, dst = np.array([0], np.int32), np.array([1], np.int32)
    alloc, free = sim.tensor_lifetimes(2, src, dst, [0, 1], 2, st, en, arr)
    np.testing.assert_allclose(alloc, [[0, 5], [-1, 5]])
    np.testing.assert_allclose(free, [[5, 7], [-1, 7]])


def test_peak_memory_fork_join_and_bounds():
    """a feeds b (same device) and c (other device); d joins them on device 0.  Checked against the
    intervals written out by hand, and against bounds that hold for any graph."""
    #      a(0) cost 1 size 2;  b(0) cost 4 size 3;  c(1) cost 1 size 5;  d(0) cost 1 size 7; bandwidth 1
    r, st, en, arr, peak = _mem(4, [(0, 1), (0, 2), (1, 3), (2, 3)], [1, 4, 1, 1], [2, 3, 5, 7],
                                [0, 0, 1, 0], 2)
    # a: [0,1); b: [1,5); transfer a->dev1: [1,3); c on dev1: [3,4); transfer c->dev0: [4,9); d: [9,10)
    np.testing.assert_array_equal(st, [0, 1, 3, 9])
    np.testing.assert_array_equal(en, [1, 5, 4, 10])
    assert arr[0, 1] == 3 and arr[2, 0] == 9 and r == 10
    # device 0: a [0,5) (b, its consumer, ends at 5), b [1,10), copy of c [9,10), d [9,10)
    #           t=0: 2; t=1: 2+3; t=9: 3+5+7 = 15
    # device 1: copy of a [3,4), c [3,9) (until its transfer has arrived): t=3: 2+5 = 7
    np.testing.assert_allclose(peak, [15.0, 7.0])
    rng = np.random.default_rng(5)
    for seed in range(6):
        n = 14
        src, dst = tiny_random_dag(np.random.default_rng(seed), n, 0.3)
        cost = rng.integers(1, 5, n).astype(np.float32)
        size = rng.integers(1, 9, n).astype(np.float32)
        D = 3
        placement = rng.integers(0, D, n)
        r, st, en, arr = sim.timeline(n, src, dst, cost, size, placement, D, 0.5)
        peak = sim.peak_memory(n, src, dst, size, placement, D, st, en, arr)
        alloc, free = sim.tensor_lifetimes(n, src, dst, placement, D, st, en, arr)
        for d in range(D):
            on = placement == d
            copies = alloc[:, d] >= 0
            assert peak[d] >= (size[on].max() if on.any() else 0.0)        # an output is live while its op runs
            assert peak[d] <= size[copies].sum() + 1e-9                       # never more than everything at once
            assert (free[copies, d] >= alloc[copies, d]).all()
        assert (en >= st).all() and (st >= 0).all()


def test_penalised_runtime_formula():
    """R(p) = r below the limit, r + c (m - M) above it, c = 2 by default (appendix, "Reward")."""
    assert sim.penalised_runtime(3.0, 10.0, 10.7) == 3.0
    assert sim.penalised_runtime(3.0, 10.7, 10.7) == 3.0
    assert abs(sim.penalised_runtime(3.0, 12.7, 10.7) - 7.0) < 1e-12
    assert abs(sim.penalised_runtime(3.0, 12.7, 10.7, c=0.5) - 4.0) < 1e-12
