"""CPU oracle for the runtime simulator of a placement (Appendix, "Simulator").

TEST INFRASTRUCTURE ONLY: imported by tests/; shares no code with the HIP library.

What the paper fixes: every device d has a FIFO queue of runnable operations and a FIFO
queue of output tensors waiting to leave d; a device runs one operation at a time and its
bus carries one tensor at a time, transfers overlap with compute; an operation is runnable on
its device once all its parents have finished and their outputs have arrived there; an
event-driven loop with op-done, transfer-done and wakeup events produces the timeline; the
simulated run time is the timestamp of the last op-done event; a transfer takes
size / bandwidth.

Readings where the paper is silent:
 * one run time per operation (the synthetic workloads have one cost per node, so all devices
   are alike);
 * transfers per output tensor: the printed op-done handler walks the children of the finished
   operation and enqueues the output for every child that sits on another device, and the
   printed transfer-done handler then looks at the one operation that takes the tensor as its
   input.  Read literally, an output needed by k children on one remote device crosses the bus
   k times (`per_child=True`).  The default (`per_child=False`) sends it once per destination
   device and releases every child waiting there when it arrives: a tensor that is on a device
   is there for all its consumers, which is how the framework whose graphs the paper places
   moves tensors between devices.  The two differ whenever several children of one operation
   share a remote device; both are kept, pinned by hand-computed timelines, and the build's
   other pieces (rewards, benchmarks) use the default;
 * operations without parents are queued in ascending node id at time 0; the children of a
   finished operation are visited in ascending node id;
 * events are taken in order of (timestamp, creation number); after every event the free
   devices 0..D-1 with a non-empty queue are started first, then the free buses 0..D-1
   (these are the paper's wakeups);
 * timestamps are float32, formed as start + cost and start + size * (1 / bandwidth) with one
   rounding per operation: the event order is an integer decision taken in this precision
   on both sides, so the two timelines are identical event by event;
 * peak memory (the paper only says that the start and end timestamps of the operations and the
   tensor sizes are used to predict it; the model below is the reading taken here): the output of
   an operation occupies its own device from the operation's START until the latest of its own
   end, the end of its last consumer on that device and the arrival of its last outgoing
   transfer; on every other device that consumes it, a copy lives from the transfer's arrival
   until the end of its last consumer there.  Intervals are half-open [alloc, free): what is
   freed at time t does not count at t.  A device's peak is the largest sum of live sizes at
   any allocation time (the sum can only grow at an allocation); m is the largest peak over
   the devices, and the reward's memory-penalised run time is the appendix's
   R(p) = r if m <= M else r + c (m - M), c = 2 in the paper.
"""
from __future__ import annotations

from collections import deque

import numpy as np

F = np.float32


def simulate(n, src, dst, cost, out_bytes, placement, D, inv_bandwidth, trace=None, per_child=False):
    """Run time of one placement of one graph.  src/dst: edges (parent, child), graph-local
    ids.  Returns (runtime float32, n_events).  `trace`, if a list, receives
    (kind, node, device, timestamp) per processed event.  per_child: one transfer per child on
    another device (the printed handlers) instead of one per destination device."""
    src = np.asarray(src, dtype=np.int64)
    dst = np.asarray(dst, dtype=np.int64)
    cost = np.asarray(cost, dtype=F)
    out_bytes = np.asarray(out_bytes, dtype=F)
    placement = np.asarray(placement, dtype=np.int64)
    inv_bw = F(inv_bandwidth)
    children = [[] for _ in range(n)]
    pend = np.zeros(n, dtype=np.int64)
    for u, v in sorted(zip(src.tolist(), dst.tolist())):
        children[u].append(v)              # ascending child id
        pend[v] += 1
    q_op = [deque() for _ in range(D)]
    q_tr = [deque() for _ in range(D)]
    ev = {}                                # slot -> (time, seq, node, dest): slot d = device d, D + d = bus d
    seq = 0
    for v in range(n):
        if pend[v] == 0:
            q_op[placement[v]].append(v)

    def wake(now):
        nonlocal seq
        for d in range(D):
            if d not in ev and q_op[d]:
                o = q_op[d].popleft()
                ev[d] = (F(now + cost[o]), seq, o, -1)
                seq += 1
                if trace is not None:
                    trace.append(("start", o, d, float(now)))
        for d in range(D):
            if D + d not in ev and q_tr[d]:
                o, dc, child = q_tr[d].popleft()
                ev[D + d] = (F(now + F(out_bytes[o] * inv_bw)), seq, o, (dc, child))
                seq += 1

    wake(F(0.0))
    last = F(0.0)
    n_events = 0
    while ev:
        slot = min(ev, key=lambda s: (ev[s][0], ev[s][1]))
        now, _, o, dc = ev.pop(slot)
        n_events += 1
        if slot < D:                       # op-done of o on device slot
            d = slot
            last = now
            if trace is not None:
                trace.append(("op", o, d, float(now)))
            sent = set()
            for c in children[o]:
                pc = int(placement[c])
                if pc == d:
                    pend[c] -= 1
                    if pend[c] == 0:
                        q_op[pc].append(c)
                elif per_child:
                    q_tr[d].append((o, pc, c))          # one crossing for this child alone
                elif pc not in sent:
                    sent.add(pc)
                    q_tr[d].append((o, pc, -1))         # one crossing for every child on pc
        else:                              # transfer-done: o's output has arrived on device dc
            dc, child = dc
            if trace is not None:
                trace.append(("tr", o, dc, float(now)))
            for c in ([child] if per_child else children[o]):
                if int(placement[c]) == dc:
                    pend[c] -= 1
                    if pend[c] == 0:
                        q_op[dc].append(c)
        wake(now)
    assert (pend == 0).all(), "an operation never became runnable"
    return last, n_events


def timeline(n, src, dst, cost, out_bytes, placement, D, inv_bandwidth, per_child=False):
    """The simulated timeline: (runtime, op_start [n], op_end [n], arrival [n, D]) with
    arrival[v, d] = time at which v's output reached device d over the bus (-1: it never went
    there).  float32 timestamps as produced by `simulate`.  With per_child an output may reach a
    device several times: arrival is then a pair (first [n, D], last [n, D])."""
    trace = []
    runtime, _ = simulate(n, src, dst, cost, out_bytes, placement, D, inv_bandwidth, trace, per_child)
    op_start = np.full(n, -1.0, dtype=F)
    op_end = np.full(n, -1.0, dtype=F)
    first = np.full((n, D), -1.0, dtype=F)
    last = np.full((n, D), -1.0, dtype=F)
    for kind, o, d, t in trace:
        if kind == "start":
            op_start[o] = F(t)
        elif kind == "op":
            op_end[o] = F(t)
        else:
            if first[o, d] < 0:
                first[o, d] = F(t)
            last[o, d] = F(t)                 # events come in time order
    return runtime, op_start, op_end, ((first, last) if per_child else last)


def tensor_lifetimes(n, src, dst, placement, D, op_start, op_end, arrival):
    """alloc [n, D], free [n, D]: the interval during which a copy of v's output occupies device d
    (-1, -1: no copy there), by the reading stated in the module docstring.  `arrival` is [n, D],
    or (first, last) when an output may cross to a device more than once (per-child transfers):
    the copy is there from the first arrival, the source waits for the last."""
    placement = np.asarray(placement, dtype=np.int64)
    arrival, arrival_last = arrival if isinstance(arrival, tuple) else (arrival, arrival)
    alloc = np.full((n, D), -1.0)
    free = np.full((n, D), -1.0)
    last_use = np.full((n, D), -1.0)          # end of the last consumer of v on device d
    for u, c in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
        pc = int(placement[c])
        last_use[u, pc] = max(last_use[u, pc], float(op_end[c]))
    for v in range(n):
        d = int(placement[v])
        alloc[v, d] = float(op_start[v])
        free[v, d] = max(float(op_end[v]), last_use[v, d])
        for o in range(D):
            if o != d and arrival[v, o] >= 0:
                free[v, d] = max(free[v, d], float(arrival_last[v, o]))   # the source stays until it has been sent
                alloc[v, o] = float(arrival[v, o])
                free[v, o] = max(float(arrival[v, o]), last_use[v, o])
    return alloc, free


def peak_memory(n, src, dst, out_bytes, placement, D, op_start, op_end, arrival) -> np.ndarray:
    """peak [D] in float64: for every device the largest sum, over all allocation times t, of the
    sizes of the copies with alloc <= t < free."""
    alloc, free = tensor_lifetimes(n, src, dst, placement, D, op_start, op_end, arrival)
    size = np.asarray(out_bytes, dtype=np.float64)
    peak = np.zeros(D)
    for d in range(D):
        have = alloc[:, d] >= 0
        a, f, s = alloc[have, d], free[have, d], size[have]
        for t in a:
            live = s[(a <= t) & (t < f)].sum()
            peak[d] = max(peak[d], live)
    return peak


def penalised_runtime(r, m, M, c=2.0):
    """R(p) of the appendix ("Reward"): r if m <= M, else r + c (m - M)."""
    return float(r) if m <= M else float(r) + c * (float(m) - float(M))
