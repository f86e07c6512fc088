"""Pins for the simulator oracle (oracle/simulator.py): closed forms on small graphs, bounds
that any valid schedule obeys, and the FIFO and overlap rules the paper states."""
import numpy as np
import pytest

from oracle import simulator as sim
from workloads import make_workload, tiny_random_dag

BW = 1.0 / 1024.0     # seconds per byte in these tests is 1/1024: sizes in KiB become seconds


def run(n, edges, cost, size, place, D, inv_bw=BW, trace=None):
    src = [e[0] for e in edges]
    dst = [e[1] for e in edges]
    return sim.simulate(n, src, dst, cost, size, place, D, inv_bw, trace)


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


def test_device_queue_is_fifo_in_ready_order():
    # device 1 gets op 3 (ready at 1) before op 2 (ready at 2): FIFO by readiness, not by id
    trace = []
    run(4, [(0, 2), (1, 3)], [2, 1, 5, 5], [0, 0, 0, 0], [0, 0, 0, 0], 1, trace=trace)
    # single device: 0 (0..2), 1 (2..3), then 2 was queued at t=2, 3 at t=3
    assert [t[1] for t in trace] == [0, 1, 2, 3]
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
