#!/usr/bin/env python3
"""Benchmark of the policy forward pass on one MI355X.

A step is one pass of the whole hot path (features, both message-passing sweeps, pooling,
policy head) over one batch of synthetic graphs, called through the C ABI with all inputs
resident in HBM.  Each step uses a different pre-generated episode state (placement,
current node, visited flags).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload nasnet]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
N_STATES = 8
CPU_SAMPLE_GRAPHS = {"random32": 1, "layered200": 64, "inception": 128, "nmt": 64, "nasnet": 256}


def sweep_algorithmic_bytes(n_tot: int, e_tot: int, H: int) -> int:
    """Bytes one sweep launch (both directions) must move: per node and direction the state
    is read and written once and its message written once (3 x 4H), every edge's message is
    read once (4H), plus the bucket order, CSR offsets and neighbour ids."""
    return 2 * n_tot * (12 * H + 8) + 2 * e_tot * (4 * H + 4)


def path_algorithmic_bytes(n_tot: int, e_tot: int, H: int) -> int:
    """The whole path: the sweeps, one read of [td;bu] in pooling (8H), raw features, placement
    and flags: 4H (8 + 2 deg) per node plus indices."""
    return sweep_algorithmic_bytes(n_tot, e_tot, H) + n_tot * (8 * H + 12 + 4 + 2)


SWEEP_SOURCES = ("kernels_mfma.hip", "plan.cpp", "sweep_plan.h")
WGRAD_SOURCES = ("kernels_backward.hip",)
POOL_SOURCES = ("kernels_pool_mfma.hip",)


def csrc_digest(sources=SWEEP_SOURCES) -> str:
    """sha256 over the sources of a kernel (by default the dominant one: the sweep kernel, its
    gather plan and the shared declarations): ties a stored counter measurement to the kernel it
    was taken on."""
    import hashlib
    h = hashlib.sha256()
    for name in sources:
        h.update(name.encode())
        h.update(open(os.path.join(ROOT, "paper_1906_08879_amd", "csrc", name), "rb").read())
    return h.hexdigest()


def measured_traffic(workload: str, batch: int, key: str = "sweep_traffic_bytes_per_launch",
                     digest_key: str = "source_sha256", sources=SWEEP_SOURCES):
    """HBM bytes (per sweep launch by default; per gradient step for the weight-gradient stage)
    from the stored rocprofv3 counter summary, or None when there is none for this workload or
    the kernels have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}_B{batch}.txt")
    if not os.path.exists(path):
        return None
    rec = {}
    for line in open(path):
        if not line.startswith("#") and ":" in line:
            k, v = line.split(":", 1)
            rec[k.strip()] = v.strip()
    if rec.get(digest_key) != csrc_digest(sources) or key not in rec:
        return None
    return int(rec[key])


def forward_only(pl, torch, w, steps: int, warmup: int) -> dict:
    """ms per forward pass of workload `w` (one state), with its depth and stage times."""
    import numpy as np
    dev = torch.device("cuda:0")
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    f = torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev)
    p = torch.from_numpy(np.ascontiguousarray(w.placement, dtype=np.int32)).to(dev)
    c = torch.from_numpy(np.ascontiguousarray(w.cur_node, dtype=np.int32)).to(dev)
    logits = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
    for _ in range(warmup):
        pl.embed_forward(g, f, p, c, wt, logits)
    torch.cuda.synchronize()
    g.profile_enable(True)
    g.profile_read(reset=True)
    t0 = time.perf_counter()
    for _ in range(steps):
        pl.embed_forward(g, f, p, c, wt, logits)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    stages = g.profile_read(reset=True)
    g.profile_enable(False)
    sweep = stages["sweep"][0] / max(1, stages["sweep"][1])
    out = {"B": int(w.B), "N_tot": int(w.n_tot), "H": w.H, "ms_per_step": round(1e3 * dt, 4),
           "graph_steps_per_s": round(w.B / dt, 1), "levels": int(g.max_depth),
           "sweep_ms": round(sweep, 4), "us_per_level": round(1e3 * sweep / max(1, int(g.max_depth)), 3),
           "stage_ms": {k: round(v[0] / v[1], 4) for k, v in stages.items() if v[1]}}
    g.close()
    wt.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="nasnet")
    ap.add_argument("--batch", type=int, default=None, help="override the number of graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    # architecture variants (the headline is the default of each): sweeps per direction, layers
    # per network, pooling per (set, device) or per set, one pooled set instead of three
    ap.add_argument("--k-sweeps", type=int, default=1)
    ap.add_argument("--n-layers", type=int, default=2)
    ap.add_argument("--group-by-device", type=int, default=1, choices=(0, 1))
    ap.add_argument("--single-set", type=int, default=0, choices=(0, 1))
    ap.add_argument("--grad-steps", type=int, default=4, help="timed reverse passes (reported beside the headline)")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the short forward-only runs of the other configurations")
    ap.add_argument("--copy-probe", action="store_true",
                    help="run a plain 1 GiB device copy five times and exit (reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on ONE GPU; the path shards over the batch of "
              "independent graphs and no multi-GPU figure is produced (--gpus must be 1).",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    if args.copy_probe:
        n = 1 << 28                                     # 2^28 floats = 1 GiB read, 1 GiB written
        a = torch.ones(n, dtype=torch.float32, device="cuda:0")
        b = torch.empty_like(a)
        for _ in range(5):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"copy_probe": True, "bytes_read_per_copy": 4 * n, "bytes_written_per_copy": 4 * n,
                          "copies": 5}))
        return 0
    import paper_1906_08879_amd as pl
    from workloads import make_workload, make_states

    if not os.path.exists(pl.library_path()):
        from paper_1906_08879_amd.build import build
        build()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")

    w = make_workload(args.workload, B=args.batch, k_sweeps=args.k_sweeps, n_layers=args.n_layers,
                      group_by_device=args.group_by_device)
    w.single_set = args.single_set
    placement, cur, done = make_states(w, N_STATES)
    t_build = time.perf_counter()
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    layout_build_ms = 1e3 * (time.perf_counter() - t_build)     # host: CSR, levels, buckets (once per batch)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype,
                    w.single_set)
    feats = []
    for s in range(N_STATES):
        f = np.array(w.node_feats, dtype=np.float32, copy=True)
        f[:, 2] = done[s]
        feats.append(torch.from_numpy(f).to(dev))
    t_place = [torch.from_numpy(placement[s]).to(dev) for s in range(N_STATES)]
    t_cur = [torch.from_numpy(cur[s]).to(dev) for s in range(N_STATES)]
    logits = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def step(i):
        s = i % N_STATES
        pl.embed_forward(g, feats[s], t_place[s], t_cur[s], wt, logits, stream=stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    g.profile_enable(True)
    g.profile_read(reset=True)
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    stages = g.profile_read(reset=True)
    g.profile_enable(False)
    assert torch.isfinite(logits).all(), "non-finite logits in the timed run"

    ms_per_step = 1e3 * elapsed / args.steps
    steps_per_s = w.B * args.steps / elapsed
    stage_ms = {k: v[0] / v[1] for k, v in stages.items() if v[1]}
    sweep_ms, sweep_launches = stages["sweep"]
    launches_per_step = max(1, w.k_sweeps)
    default_variant = (args.k_sweeps, args.n_layers, args.group_by_device, args.single_set) == (1, 2, 1, 0)
    avg_launch_ms = sweep_ms / max(1, sweep_launches) / launches_per_step
    alg = sweep_algorithmic_bytes(w.n_tot, w.e_tot, w.H)
    achieved = alg / (avg_launch_ms * 1e-3) / 1e9 if avg_launch_ms > 0 else 0.0
    roofline = {"kernel": "sweep (message passing, both directions)", "bound": "hbm",
                "achieved": round(achieved, 2), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 5),
                "traffic": measured_traffic(args.workload, int(w.B)) if default_variant else None,
                "algorithmic_bytes_per_launch": alg, "avg_launch_ms": round(avg_launch_ms, 5),
                "path_algorithmic_bytes_per_step": path_algorithmic_bytes(w.n_tot, w.e_tot, w.H),
                "path_frac": round(path_algorithmic_bytes(w.n_tot, w.e_tot, w.H)
                                   / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 5),
                # what actually bounds the sweep: one dependent step per level of the deepest graph
                "levels": int(g.max_depth),
                "us_per_level": round(1e3 * avg_launch_ms / max(1, int(g.max_depth)), 4)}

    # the second stage, pooling: one read of every node's [td ; bu] (8H bytes) and its flags
    pool_alg = int(w.n_tot) * (8 * w.H + 6)
    pool_ms = stage_ms.get("pool", 0.0)
    pool_roofline = {"kernel": "pooling (sort by set and device + l_i of every node, summed per key)",
                     "bound": "hbm", "achieved": round(pool_alg / (pool_ms * 1e-3) / 1e9, 2) if pool_ms > 0 else 0.0,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(pool_alg / (pool_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 5) if pool_ms > 0 else 0.0,
                     "traffic": (measured_traffic(args.workload, int(w.B), "pool_traffic_bytes_per_launch", "pool_sha256", POOL_SOURCES)
                                 if default_variant else None),
                     "algorithmic_bytes_per_launch": pool_alg, "avg_stage_ms": round(pool_ms, 5)}

    # a plain device copy of 1 GiB on the same GPU: what the published peak means in practice here
    cp_a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    cp_b = torch.empty_like(cp_a)
    cp_b.copy_(cp_a)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(5):
        cp_b.copy_(cp_a)
    torch.cuda.synchronize()
    roofline["device_copy_GBs"] = round(5 * 2 * 4 * (1 << 28) / (time.perf_counter() - t0) / 1e9, 1)
    del cp_a, cp_b

    # the same path driven as an episode (Section 2.1): forward pass + on-device transition per
    # step, enqueued without host synchronisation; reported beside the headline, not in it
    from workloads import make_episode
    ep_steps = 16
    order, uniforms, placement0 = make_episode(w, ep_steps)
    f0 = np.array(w.node_feats, dtype=np.float32, copy=True)
    f0[:, 2] = 0.0
    cur0 = np.array([order[w.node_off[b]] for b in range(w.B)], dtype=np.int32)
    e_f, e_p, e_c, e_o, e_u = (torch.from_numpy(np.ascontiguousarray(x)).to(dev)
                               for x in (f0, placement0, cur0, order, uniforms))
    e_act = torch.empty((ep_steps, w.B), dtype=torch.int32, device=dev)
    pl.episode_run(g, wt, e_f, e_p, e_c, e_o, e_u, 0, 2, logits, False, e_act, None, stream=stream)
    e_f.copy_(torch.from_numpy(f0)); e_p.copy_(torch.from_numpy(placement0)); e_c.copy_(torch.from_numpy(cur0))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    pl.episode_run(g, wt, e_f, e_p, e_c, e_o, e_u, 0, ep_steps, logits, False, e_act, None, stream=stream)
    torch.cuda.synchronize()
    ep_elapsed = time.perf_counter() - t0
    episode = {"steps": ep_steps, "ms_per_step": round(1e3 * ep_elapsed / ep_steps, 4),
               "graph_steps_per_s": round(w.B * ep_steps / ep_elapsed, 2),
               "what": "forward pass + sampled on-device transition per step, from the trivial placement"}

    # the run-time simulator of the paper's appendix on the same batch (the reward of an episode
    # needs one run per episode, or one per step with intermediate rewards); beside the headline
    sim_rt = torch.empty((w.B,), dtype=torch.float32, device=dev)
    sim_ev = torch.empty((w.B,), dtype=torch.int32, device=dev)
    inv_bw = 5e-5
    pl.simulate_runtime(g, w.D, feats[0], t_place[0], inv_bw, sim_rt, sim_ev, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    sim_reps = 5
    for i in range(sim_reps):
        pl.simulate_runtime(g, w.D, feats[0], t_place[i % N_STATES], inv_bw, sim_rt, sim_ev, stream=stream)
    torch.cuda.synchronize()
    sim_elapsed = (time.perf_counter() - t0) / sim_reps
    sim_rew = torch.empty((w.B,), dtype=torch.float32, device=dev)
    pl.simulate_reward(g, w.D, feats[0], t_place[0], inv_bw, 1e12, 2.0, sim_rew, stream=stream)   # allocates
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(sim_reps):
        pl.simulate_reward(g, w.D, feats[0], t_place[i % N_STATES], inv_bw, 1e12, 2.0, sim_rew, stream=stream)
    torch.cuda.synchronize()
    rew_elapsed = (time.perf_counter() - t0) / sim_reps
    simulator = {"ms_per_batch": round(1e3 * sim_elapsed, 4),
                 "ms_per_batch_with_peak_memory": round(1e3 * rew_elapsed, 4),
                 "placements_per_s": round(w.B / sim_elapsed, 1),
                 "events_per_s": round(float(sim_ev.sum().item()) / sim_elapsed, 1),
                 "what": "event-driven run-time simulation of one placement per graph (one wave per graph)"}

    # one REINFORCE term (appendix "REINFORCE Algorithm", Eq. 1) for the same batch: forward pass +
    # reverse pass, gradient summed over the batch; beside the headline, not in it
    n_par = pl.weights_count(w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    gradient = None
    if args.grad_steps > 0:
        g_act = torch.from_numpy(np.random.default_rng(0).integers(0, w.D, w.B).astype(np.int32)).to(dev)
        g_coef = torch.from_numpy(np.random.default_rng(1).normal(0, 1, w.B).astype(np.float32)).to(dev)
        g_grad = torch.empty((n_par,), dtype=torch.float32, device=dev)
        pl.policy_gradient(g, feats[0], t_place[0], t_cur[0], wt, g_act, g_coef, g_grad, logits, stream=stream)
        torch.cuda.synchronize()
        g.profile_enable(True)
        g.profile_read(reset=True)
        t0 = time.perf_counter()
        for i in range(args.grad_steps):
            s_ = i % N_STATES
            pl.policy_gradient(g, feats[s_], t_place[s_], t_cur[s_], wt, g_act, g_coef, g_grad, logits,
                               accumulate=i > 0, stream=stream)
        torch.cuda.synchronize()
        gr_elapsed = (time.perf_counter() - t0) / max(1, args.grad_steps)
        gr_stages = g.profile_read(reset=True)
        g.profile_enable(False)
        assert torch.isfinite(g_grad).all(), "non-finite gradient in the timed run"
        gradient = {"ms_per_step": round(1e3 * gr_elapsed, 4), "steps": args.grad_steps,
                    "graph_steps_per_s": round(w.B / gr_elapsed, 2), "parameters": int(n_par),
                    # per step: a stage may be timed in several intervals of one call
                    "stage_ms": {k: round(v[0] / max(1, args.grad_steps), 4) for k, v in gr_stages.items() if v[1]},
                    "what": "forward pass + reverse pass (log-probability gradient of one decision per "
                            "graph, summed over the batch)"}
        # the reverse pass's largest stage: every layer's weight gradient is a contraction over rows,
        # 2 R I J flops each, that reads its two operands (R x I inputs, R x J deltas, fp32) once:
        # projection (F inputs), 2 directions x (f, g) x L layers of H x H per sweep, l (2H x H, then
        # H x H) over the nodes of the three sets (all nodes but the current ones).  With each operand
        # split into three bf16 parts and six products kept, the matrix cores have 6 x those flops to
        # do at the bf16 rate (less time than the operands take to arrive): the stage is priced
        # against HBM.
        wg_ms = gradient["stage_ms"].get("bw_wgrad")
        if wg_ms:
            n, H, L, F = float(w.n_tot), float(w.H), float(w.n_layers), float(w.D + 4)
            n_set = n - w.B
            flops = 2.0 * H * (n * F + n * 4.0 * L * H * w.k_sweeps + n_set * (2.0 * H + (L - 1.0) * H))
            alg = 4.0 * (n * (F + H) + n * 4.0 * L * 2.0 * H * w.k_sweeps
                         + n_set * (3.0 * H + (L - 1.0) * 2.0 * H))
            gbs = alg / (wg_ms * 1e-3) / 1e9
            gradient["roofline"] = {"kernel": "weight-gradient contractions (bf16 matrix cores, operands split "
                                              "in three parts) + slab sums",
                                    "bound": "hbm", "achieved": round(gbs, 2), "peak": HBM_PEAK_GBS,
                                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                                    "algorithmic_bytes_per_step": int(alg), "flops_per_step": int(flops),
                                    "matrix_core_tflops": round(6.0 * flops / (wg_ms * 1e-3) / 1e12, 1),
                                    "traffic": measured_traffic(args.workload, int(w.B),
                                                                "wgrad_stage_traffic_bytes_per_step",
                                                                "backward_sha256", WGRAD_SOURCES)
                                    if default_variant else None}

    # the other configurations, forward pass only, a few steps each: what bounds them is the number
    # of dependent level steps (levels x time per level), not bandwidth
    other = None
    if default_variant and args.batch is None and not args.no_other_workloads:
        other = {}
        for name in ("random32", "layered200", "inception", "nmt", "nasnet"):
            if name == args.workload:
                continue
            other[name] = forward_only(pl, torch, make_workload(name), 20, 3)

    # a batch of rollouts of ONE graph (the batch shape of the REINFORCE baseline): the layout is
    # built once and the sweep kernel's plan is shared by all copies
    replicated = None
    if default_variant and args.batch is None and not args.no_other_workloads:
        one = make_workload(args.workload, B=1)
        t0 = time.perf_counter()
        g_rep = pl.GraphBatch(int(one.n_nodes[0]), int(one.n_edges[0]), one.edge_src, one.edge_dst, replicate=int(w.B))
        rep_build_ms = 1e3 * (time.perf_counter() - t0)
        n1 = int(one.n_nodes[0])
        rng = np.random.default_rng(5)
        r_f = torch.from_numpy(np.tile(np.asarray(one.node_feats, np.float32), (int(w.B), 1))).to(dev)
        r_p = torch.from_numpy(rng.integers(0, w.D, n1 * int(w.B)).astype(np.int32)).to(dev)
        r_c = torch.from_numpy(rng.integers(0, n1, int(w.B)).astype(np.int32)).to(dev)
        for _ in range(3):
            pl.embed_forward(g_rep, r_f, r_p, r_c, wt, logits)
        torch.cuda.synchronize()
        g_rep.profile_enable(True)
        g_rep.profile_read(reset=True)
        t0 = time.perf_counter()
        for _ in range(10):
            pl.embed_forward(g_rep, r_f, r_p, r_c, wt, logits)
        torch.cuda.synchronize()
        rep_ms = 1e2 * (time.perf_counter() - t0)
        rep_st = g_rep.profile_read(reset=True)
        replicated = {"rollouts": int(w.B), "nodes_per_graph": n1, "levels": int(g_rep.max_depth),
                      "layout_build_ms": round(rep_build_ms, 2), "ms_per_step": round(rep_ms, 4),
                      "stage_ms": {k: round(v[0] / v[1], 4) for k, v in rep_st.items() if v[1]},
                      "what": "B rollouts of the first graph of the workload, one shared layout and gather plan"}
        g_rep.close()

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle
        n_s = min(w.B, CPU_SAMPLE_GRAPHS.get(args.workload, 32))
        ws = make_workload(args.workload, B=n_s, k_sweeps=args.k_sweeps, n_layers=args.n_layers,
                           group_by_device=args.group_by_device)
        ws.single_set = args.single_set
        threads = min(16, os.cpu_count() or 1)
        oracle.load()
        t0 = time.perf_counter()
        oracle.forward_workload(ws, n_threads=threads, want_emb=False)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": round(n_s / dt, 3), "unit": "graph-steps/s", "cores": threads,
                        "kind": "oracle",
                        "sample": f"one forward of the first {n_s} graphs of '{args.workload}' "
                                  f"({int(ws.n_tot)} nodes), float64 C oracle, {dt:.2f} s wall",
                        "node_embeddings_per_s": round(ws.n_tot / dt, 1)}
        # the same oracle on one thread, on the layered-DAG configuration (its whole batch)
        wl = make_workload("layered200")
        t0 = time.perf_counter()
        oracle.forward_workload(wl, n_threads=1, want_emb=False)
        cpu_baseline["one_thread_layered200_graph_steps_per_s"] = round(wl.B / (time.perf_counter() - t0), 2)
        # the oracles of the rows beside the headline, on bounded samples (one graph each)
        from oracle import gradient as og, simulator as osim
        w1 = make_workload(args.workload, B=1, k_sweeps=args.k_sweeps, n_layers=args.n_layers,
                           group_by_device=args.group_by_device)
        w1.single_set = args.single_set
        t0 = time.perf_counter()
        osim.simulate(int(w1.n_nodes[0]), w1.edge_src, w1.edge_dst, w1.node_feats[:, 0], w1.node_feats[:, 1],
                      w1.placement, w1.D, np.float32(inv_bw))
        simulator["cpu_oracle_placements_per_s"] = round(1.0 / (time.perf_counter() - t0), 2)
        if gradient is not None:
            t0 = time.perf_counter()
            og.gradient_workload(w1, [0], [1.0])
            gradient["cpu_oracle_graph_steps_per_s"] = round(1.0 / (time.perf_counter() - t0), 3)

    out = {
        "metric": "policy forward steps/sec (graphs x steps)",
        "value": round(steps_per_s, 2), "unit": "graph-steps/s",
        "node_embeddings_per_s": round(w.n_tot * args.steps / elapsed, 1),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if w.weight_dtype == "fp32" else "f32 (bf16 weights)",
        "data": "synthetic",
        "config": {"workload": args.workload, "B": int(w.B), "N_tot": int(w.n_tot),
                   "E_tot": int(w.e_tot), "D": w.D, "H": w.H, "n_layers": w.n_layers,
                   "k_sweeps": w.k_sweeps, "group_by_device": w.group_by_device,
                   "single_set": w.single_set, "max_depth": int(g.max_depth),
                   "weight_dtype": w.weight_dtype, "states": N_STATES},
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "layout_build_ms": round(layout_build_ms, 2),
        "roofline": roofline,
        "pool_roofline": pool_roofline,
        "other_workloads": other,
        "replicated_batch": replicated,
        "episode": episode,
        "simulator": simulator,
        "gradient": gradient,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))
    g.close()
    wt.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
