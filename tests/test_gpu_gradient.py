"""GPU parity of pl_policy_gradient (appendix "REINFORCE Algorithm", Eq. 1) against the float64
autograd oracle on the same seeded inputs, through the C ABI.

Bar: for every layer's block of the gradient (matrix and bias), the largest error is at most
GRAD_RTOL times the largest entry of the oracle's block plus GRAD_ATOL times the largest entry of
the whole gradient.  A weight's gradient is an fp32 sum over up to ~10^6 rows of products of two
fp32 chains (~10^3 dependent levels each) whose values differ from float64 by ~1e-6 relative, so
single entries formed by cancellation cannot meet a bound relative to their own size; the block's
largest entry sets the scale, as the row's largest logit does for the forward pass.  2e-5 is a
fifth of the forward pass's 1e-4; measured worst case: 0.08 of the bound."""
import numpy as np
import pytest

import oracle
from oracle import gradient as og
from gpu_common import custom_workload, run_gradient, assert_logits_close
from workloads import make_workload

pytestmark = pytest.mark.gpu

GRAD_RTOL, GRAD_ATOL = 2e-5, 2e-7
# per output unit the absolute term is 5e-7 of the gradient's largest entry: a column's entries are
# sums over all nodes like the block's, so their rounding errors follow the gradient's scale, not
# the column's own (measured worst case 0.4 of this bound)
GRAD_ATOL_UNIT = 5e-7


def assert_grad_close(got, ref, w, what):
    """Per layer block: max error <= GRAD_RTOL x the block's largest entry + GRAD_ATOL x the
    gradient's largest entry; and the same per output unit (column of a weight matrix, with the
    column's own largest entry), so that an error confined to one unit of a layer cannot hide
    behind the block's scale."""
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    slices, total = og.layer_slices(w.D, w.H, w.n_layers, w.group_by_device)
    shapes = {name: (i, o) for name, i, o in og.layer_shapes(w.D, w.H, w.n_layers, w.group_by_device)}
    assert total == got.size == ref.size
    gmax = np.abs(ref).max()
    worst = 0.0
    for name, (ws, bs) in slices.items():
        for part, sl in (("W", ws), ("b", bs)):
            err = np.abs(got[sl] - ref[sl]).max()
            bound = GRAD_RTOL * np.abs(ref[sl]).max() + GRAD_ATOL * gmax
            worst = max(worst, err / max(bound, 1e-300))
            assert err <= bound, f"{what}: layer {name}.{part}: error {err:.3g} > {bound:.3g} (block max {np.abs(ref[sl]).max():.3g})"
        n_in, n_out = shapes[name]
        e2 = np.abs(got[ws] - ref[ws]).reshape(n_in, n_out).max(axis=0)
        col = np.abs(ref[ws]).reshape(n_in, n_out).max(axis=0)
        b2 = np.maximum(GRAD_RTOL * col + GRAD_ATOL_UNIT * gmax, 1e-300)
        j = int(np.argmax(e2 / b2))
        worst = max(worst, float(e2[j] / b2[j]))
        assert e2[j] <= b2[j], f"{what}: layer {name}, output unit {j}: error {e2[j]:.3g} > {b2[j]:.3g} (column max {col[j]:.3g})"
    return worst


def _actions_and_coeff(w, seed):
    """Half of the graphs take their least likely device (a large gradient), the rest a random one."""
    rng = np.random.default_rng(seed)
    ref = oracle.forward_workload(w, n_threads=8, want_emb=False)
    actions = rng.integers(0, w.D, w.B).astype(np.int32)
    low = np.argmin(ref["logits"], axis=1).astype(np.int32)
    pick = rng.random(w.B) < 0.5
    actions[pick] = low[pick]
    coeff = rng.normal(0, 1, w.B).astype(np.float32)
    return actions, coeff, ref


def _compare(w, what, seed=0, path=0):
    actions, coeff, fwd = _actions_and_coeff(w, seed)
    print(f"[gradient] {what}", flush=True)
    got = run_gradient(w, actions, coeff, path=path)
    ref_grad, ref_logp = og.gradient_workload(w, actions, coeff.astype(np.float64))
    assert_logits_close(got["logits"], fwd["logits"], what, 0.1)
    scale = np.abs(fwd["logits"]).max(axis=1)
    assert (np.abs(got["logp"] - ref_logp) <= 1e-4 * scale + 1e-5).all(), what
    worst = assert_grad_close(got["grad"], ref_grad, w, what)
    print(f"[gradient] {what}: worst error / bound = {worst:.3g}", flush=True)
    return got, ref_grad


@pytest.mark.parametrize("D,H,L,k,group,wd", [
    (2, 8, 2, 1, 1, "fp32"), (1, 5, 1, 1, 1, "fp32"), (16, 16, 2, 1, 1, "fp32"),
    (4, 48, 3, 1, 1, "fp32"), (3, 100, 2, 1, 0, "fp32"), (4, 32, 2, 0, 1, "fp32"),
    (8, 128, 2, 1, 1, "bf16"), (2, 256, 2, 1, 1, "fp32"), (4, 64, 4, 1, 1, "bf16"), (12, 6, 2, 1, 1, "fp32"),
    (4, 64, 1, 1, 1, "bf16"), (4, 32, 2, 1, 1, "bf16"), (4, 64, 2, 1, 1, "fp32"), (3, 128, 1, 1, 0, "bf16"),
    (5, 128, 2, 1, 1, "fp32"), (4, 32, 1, 1, 1, "fp32"),
])
def test_shapes_and_variants(D, H, L, k, group, wd):
    """Ragged batches (single nodes, edgeless graphs, wide levels) over the supported range of D,
    H, layers, pooling modes and weight formats; every parameter compared."""
    rng = np.random.default_rng(100 * D + H)
    w = custom_workload(rng, [1, 2, 40, 1, 17, 70, 3], D, H, L, k, group, wd)
    _compare(w, f"D={D} H={H} L={L} k={k} g={group} {wd}")


@pytest.mark.parametrize("name,B", [("random32", 4), ("layered200", 4), ("inception", 2), ("nmt", 2), ("nasnet", 1)])
def test_small_batches_of_the_workloads(name, B):
    _compare(make_workload(name, B=B), name)


@pytest.mark.parametrize("H,wd", [(32, "fp32"), (64, "bf16"), (128, "bf16")])
def test_dense_graphs_with_long_neighbour_lists(H, wd):
    """Nodes with dozens of parents and children: the reverse chain sums their gradients through
    the overflow lists of the chunk plan (both list walks of the kernel: one and two column tiles
    per wave)."""
    rng = np.random.default_rng(40 + H)
    w = custom_workload(rng, [150, 90, 33], 4, H, 2, 1, 1, wd, p_edge=0.4, w_scale=0.05)
    _compare(w, f"dense graphs H={H} {wd}")


@pytest.mark.parametrize("name", ["layered200", "nmt"])
def test_generic_kernels_on_matrix_core_shapes(name):
    """pl_weights_set_path(1): the generic fp32 reverse-pass kernels on shapes that normally take
    the matrix-core kernels meet the same bar, and the two paths agree closely."""
    w = make_workload(name, B=2)
    actions, coeff, _ = _actions_and_coeff(w, 3)
    ref_grad, _ = og.gradient_workload(w, actions, coeff.astype(np.float64))
    slow = run_gradient(w, actions, coeff, path=1)
    fast = run_gradient(w, actions, coeff, path=0)
    assert_grad_close(slow["grad"], ref_grad, w, name + " generic")
    assert_grad_close(fast["grad"], ref_grad, w, name + " matrix-core")
    assert np.abs(fast["grad"] - slow["grad"]).max() <= 1e-4 * np.abs(ref_grad).max()


@pytest.mark.parametrize("D,H,L,k,group,wd,path", [
    (3, 12, 2, 1, 1, "fp32", 0), (4, 32, 2, 0, 1, "fp32", 0), (4, 64, 2, 1, 1, "bf16", 0),
    (4, 64, 2, 1, 1, "bf16", 1), (5, 128, 1, 1, 0, "fp32", 0), (4, 32, 2, 2, 1, "fp32", 0),
])
def test_one_set_pooling(D, H, L, k, group, wd, path):
    """pl_model_cfg.single_set = 1 (the "simple aggregator" of Section 3.3): logits and every
    parameter's gradient; the networks of the two unused sets get exactly zero."""
    rng = np.random.default_rng(7 * D + H + k)
    w = custom_workload(rng, [1, 2, 40, 1, 17, 70, 3], D, H, L, k, group, wd)
    w.single_set = 1
    got, ref_grad = _compare(w, f"one set D={D} H={H} L={L} k={k} g={group} {wd} path={path}", path=path)
    slices, _ = og.layer_slices(D, H, L, group)
    for name, (ws, bs) in slices.items():
        if name.startswith("l_chi") or name.startswith("l_pll"):
            assert not got["grad"][ws].any() and not got["grad"][bs].any(), name
            assert not ref_grad[ws].any() and not ref_grad[bs].any(), name
    # the same inputs with the three sets give other logits: the flag reached the kernels
    w.single_set = 0
    actions, coeff, _ = _actions_and_coeff(w, 0)
    three = run_gradient(w, actions, coeff, path=path)
    assert np.abs(three["logits"] - got["logits"]).max() > 1e-6


def test_accumulation_linearity_and_rejected_states():
    rng = np.random.default_rng(5)
    w = custom_workload(rng, [30, 12, 25, 8], 4, 32)
    actions, coeff, _ = _actions_and_coeff(w, 1)
    base = run_gradient(w, actions, coeff)
    again = run_gradient(w, actions, coeff)
    np.testing.assert_array_equal(base["grad"], again["grad"])            # bitwise run to run
    start = rng.normal(0, 1, base["grad"].size).astype(np.float32)
    acc = run_gradient(w, actions, coeff, accumulate_into=start)
    np.testing.assert_allclose(acc["grad"], start + base["grad"], rtol=0, atol=1e-6 * np.abs(base["grad"]).max() + 1e-6)
    # an out-of-range action or current node contributes nothing and reports NaN
    bad_a = actions.copy()
    bad_a[1] = w.D
    bad_cur = np.array(w.cur_node, copy=True)
    bad_cur[2] = -1
    got = run_gradient(w, bad_a, coeff, cur_node=bad_cur)
    c2 = coeff.copy()
    c2[1] = 0.0
    c2[2] = 0.0
    ref_grad, _ = og.gradient_workload(w, actions, c2.astype(np.float64))
    assert_grad_close(got["grad"], ref_grad, w, "rejected states")
    assert np.isnan(got["logp"][1]) and np.isnan(got["logp"][2]) and np.isfinite(got["logp"][[0, 3]]).all()


def test_nodes_with_a_device_out_of_range_get_no_gradient_on_either_path():
    """A node whose device id is outside [0, D) is pooled nowhere, so the reverse pooling must leave
    its rows zero.  The autograd oracle has no such input; the generic kernels and the matrix-core
    kernels (whose reverse pooling walks the forward pass's tiles and never sees such a node) are
    two implementations of the same rule and must agree to the gradient bar."""
    rng = np.random.default_rng(77)
    w = custom_workload(rng, [40, 70, 17, 33], 8, 128, 2, 1, 1, "bf16")
    bad = np.array(w.placement, copy=True)
    for b in range(w.B):
        lo, hi = int(w.node_off[b]), int(w.node_off[b + 1])
        pick = [v for v in range(lo, hi) if v - lo != int(w.cur_node[b])][:3]
        bad[pick[0]] = w.D
        bad[pick[1]] = -1
    w.placement = bad
    actions = rng.integers(0, w.D, w.B).astype(np.int32)
    coeff = rng.normal(0, 1, w.B).astype(np.float32)
    fast = run_gradient(w, actions, coeff, path=0)
    slow = run_gradient(w, actions, coeff, path=1)
    assert np.isfinite(fast["grad"]).all() and np.isfinite(slow["grad"]).all()
    worst = assert_grad_close(fast["grad"], slow["grad"].astype(np.float64), w, "device out of range")
    print(f"[gradient] device out of range: matrix-core vs generic, worst error / bound = {worst:.3g}", flush=True)


@pytest.mark.parametrize("case", ["generic", "matrix-core", "nmt"])
def test_entropy_term(case):
    """Appendix A.7 "Entropy": the loss also carries beta * H(pi); gradient and entropies against the
    oracle, alone and mixed with the log-probability term; a graph without a valid current node
    adds nothing."""
    rng = np.random.default_rng(12)
    if case == "generic":
        w = custom_workload(rng, [25, 9, 40, 1], 5, 12, w_scale=0.12)
    elif case == "matrix-core":
        w = custom_workload(rng, [25, 9, 40, 1], 4, 64, 2, 1, 1, "bf16", w_scale=0.06)
    else:
        w = make_workload("nmt", B=2)
    actions, coeff, fwd = _actions_and_coeff(w, 4)
    beta = rng.uniform(0.1, 2.0, w.B).astype(np.float32)
    for c, what in ((np.zeros(w.B, np.float32), "entropy only"), (coeff, "mixed")):
        got = run_gradient(w, actions, c, entropy_coeff=beta)
        ref_grad, _, ref_ent = og.gradient_workload(w, actions, c.astype(np.float64), entropy_coeff=beta.astype(np.float64),
                                                    want_entropy=True)
        worst = assert_grad_close(got["grad"], ref_grad, w, f"{case} {what}")
        print(f"[gradient] entropy {case} {what}: worst error / bound = {worst:.3g}", flush=True)
        scale = np.abs(fwd["logits"]).max(axis=1)
        assert (np.abs(got["entropy"] - ref_ent) <= 1e-4 * scale + 1e-5).all(), (got["entropy"], ref_ent)
    bad_cur = np.array(w.cur_node, copy=True)
    bad_cur[0] = -1
    got = run_gradient(w, actions, coeff, entropy_coeff=beta, cur_node=bad_cur)
    c2, b2 = coeff.copy(), beta.copy()
    c2[0] = 0.0
    b2[0] = 0.0
    ref_grad, _ = og.gradient_workload(w, actions, c2.astype(np.float64), entropy_coeff=b2.astype(np.float64))
    assert_grad_close(got["grad"], ref_grad, w, f"{case} rejected state")
    assert np.isnan(got["entropy"][0]) and np.isfinite(got["entropy"][1:]).all()


def test_gradient_replays_from_a_hip_graph():
    """After the first call on a batch a gradient call only launches kernels (the zero fill is a
    kernel too), so it can be captured once and replayed: replays on new states, with eager work
    in between, each equal bit for bit to the eager result on the same state."""
    import torch
    import paper_1906_08879_amd as pl
    from workloads import make_states
    dev = torch.device("cuda:0")
    w = make_workload("layered200", B=8)
    placement, cur, done = make_states(w, 3)
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    n_par = pl.weights_count(w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    rng = np.random.default_rng(2)
    act = torch.from_numpy(rng.integers(0, w.D, w.B).astype(np.int32)).to(dev)
    coef = torch.from_numpy(rng.normal(0, 1, w.B).astype(np.float32)).to(dev)

    def state(s):
        f = np.array(w.node_feats, dtype=np.float32)
        f[:, 2] = done[s]
        return torch.from_numpy(f).to(dev), torch.from_numpy(placement[s]).to(dev), torch.from_numpy(cur[s]).to(dev)

    f_in, p_in, c_in = state(0)
    logits = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
    grad = torch.empty((n_par,), dtype=torch.float32, device=dev)
    eager = torch.empty_like(grad)
    pl.policy_gradient(g, f_in, p_in, c_in, wt, act, coef, eager, logits)      # first call: allocates
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        graph.capture_begin()
        pl.policy_gradient(g, f_in, p_in, c_in, wt, act, coef, grad, logits, stream=side)
        graph.capture_end()
    torch.cuda.current_stream().wait_stream(side)
    for s in (1, 2, 1):
        f, p, c = state(s)
        pl.policy_gradient(g, f, p, c, wt, act, coef, eager, logits)            # eager work between the replays
        torch.cuda.synchronize()
        f_in.copy_(f); p_in.copy_(p); c_in.copy_(c)
        grad.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        np.testing.assert_array_equal(grad.cpu().numpy(), eager.cpu().numpy())
    del graph
    g.close()
    wt.close()


def test_interleaved_handles_share_nothing():
    """Two graph batches and two weight sets of different shapes, used alternately for forward
    passes and gradients: every result equals the one computed with fresh handles."""
    import paper_1906_08879_amd as pl
    from gpu_common import run_library
    wa = make_workload("layered200", B=3)
    rng = np.random.default_rng(77)
    wb = custom_workload(rng, [30, 5, 61], 3, 64, 2, 1, 1, "bf16")
    act_a, co_a, _ = _actions_and_coeff(wa, 1)
    act_b, co_b, _ = _actions_and_coeff(wb, 2)
    alone = {"a": run_gradient(wa, act_a, co_a), "b": run_gradient(wb, act_b, co_b),
             "fa": run_library(wa, want_emb=False), "fb": run_library(wb, want_emb=False)}
    ha = (pl.GraphBatch(wa.n_nodes, wa.n_edges, wa.edge_src, wa.edge_dst),
          pl.Weights(wa.weights, wa.D, wa.H, wa.n_layers, wa.k_sweeps, wa.group_by_device, wa.weight_dtype))
    hb = (pl.GraphBatch(wb.n_nodes, wb.n_edges, wb.edge_src, wb.edge_dst),
          pl.Weights(wb.weights, wb.D, wb.H, wb.n_layers, wb.k_sweeps, wb.group_by_device, wb.weight_dtype))
    for _ in range(2):
        ga = run_gradient(wa, act_a, co_a, handles=ha)
        fb = run_library(wb, want_emb=False, handles=hb)
        gb = run_gradient(wb, act_b, co_b, handles=hb)
        fa = run_library(wa, want_emb=False, handles=ha)
        np.testing.assert_array_equal(ga["grad"], alone["a"]["grad"])
        np.testing.assert_array_equal(gb["grad"], alone["b"]["grad"])
        np.testing.assert_array_equal(fa["logits"], alone["fa"]["logits"])
        np.testing.assert_array_equal(fb["logits"], alone["fb"]["logits"])
    for h in ha + hb:
        h.close()


def test_empty_batch_is_accepted():
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    g = pl.GraphBatch([], [], [], [])
    wt = pl.Weights(np.zeros(pl.weights_count(2, 8), np.float32), 2, 8)
    z_f, z_i = torch.zeros(4, dtype=torch.float32, device=dev), torch.zeros(4, dtype=torch.int32, device=dev)
    grad = torch.full((pl.weights_count(2, 8),), 3.0, dtype=torch.float32, device=dev)
    pl.policy_gradient(g, z_f, z_i, z_i, wt, z_i, z_f, grad, z_f)
    torch.cuda.synchronize()
    assert (grad == 3.0).all()                  # nothing to add, nothing touched
    g.close()
    wt.close()


@pytest.mark.parametrize("D,H,L,k,wd", [(3, 12, 2, 2, "fp32"), (4, 32, 2, 2, "fp32"), (4, 64, 2, 3, "bf16"),
                                        (2, 128, 1, 2, "bf16"), (4, 64, 3, 2, "bf16"), (5, 128, 2, 2, "fp32")])
def test_several_sweeps(D, H, L, k, wd):
    """k >= 2 repetitions of the message passing (Section 2.2 step 2): the sweeps are differentiated
    from the last to the first with the states and messages that the forward pass copied aside;
    generic kernels, matrix-core chain, and matrix-core dense layers with the generic chain."""
    rng = np.random.default_rng(7 * H + k)
    w = custom_workload(rng, [30, 1, 12, 45], D, H, L, k, 1, wd, w_scale=0.07)
    _compare(w, f"k={k} D={D} H={H} L={L} {wd}")


def test_full_size_batch_sampled_graphs():
    """The benchmark's NASNet-like batch (256 graphs) in its launch shape; three graphs carry a
    non-zero scalar and the oracle differentiates those."""
    w = make_workload("nasnet")
    fwd = oracle.forward_workload(w, n_threads=16, want_emb=False)
    sample = [0, 101, 255]
    actions = np.argmin(fwd["logits"], axis=1).astype(np.int32)
    coeff = np.zeros(w.B, np.float32)
    coeff[sample] = [1.0, -0.5, 2.0]
    print("[gradient] nasnet full batch", flush=True)
    got = run_gradient(w, actions, coeff)
    ref_grad, ref_logp = og.gradient_workload(w, actions, coeff.astype(np.float64), only=sample)
    worst = assert_grad_close(got["grad"], ref_grad, w, "nasnet full")
    print(f"[gradient] nasnet full: worst error / bound = {worst:.3g}", flush=True)
    scale = np.abs(fwd["logits"]).max(axis=1)
    for b in sample:
        assert abs(got["logp"][b] - ref_logp[b]) <= 1e-4 * scale[b] + 1e-5
