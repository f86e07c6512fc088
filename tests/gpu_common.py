"""Shared helpers of the GPU parity tests: run the HIP library on a workload through the
C ABI and return numpy arrays; compare with the float64 oracle."""
import numpy as np

RTOL, ATOL = 1e-4, 1e-5     # fp32 logits vs the float64 oracle


def run_library(w, placement=None, cur_node=None, done=None, want_emb=True, handles=None, path=0,
                want_class=False):
    """One forward pass of workload `w` on cuda:0.  Returns dict of numpy arrays.  With
    want_class the node sets that this very pass pooled over come back as `classes`."""
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    if handles is None:
        g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
        wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device,
                        w.weight_dtype, getattr(w, "single_set", 0))
        if path:
            wt.set_path(path)
    else:
        g, wt = handles
    feats = np.array(w.node_feats, dtype=np.float32, copy=True)
    if done is not None:
        feats[:, 2] = done
    G = w.D if w.group_by_device else 1
    t_feats = torch.from_numpy(feats).to(dev)
    t_place = torch.from_numpy(np.ascontiguousarray(w.placement if placement is None else placement,
                                                    dtype=np.int32)).to(dev)
    t_cur = torch.from_numpy(np.ascontiguousarray(w.cur_node if cur_node is None else cur_node,
                                                  dtype=np.int32)).to(dev)
    logits = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    probs = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    pooled = torch.full((w.B, 3, G, w.H), float("nan"), dtype=torch.float32, device=dev)
    emb = torch.full((w.n_tot, 2 * w.H), float("nan"), dtype=torch.float32, device=dev) if want_emb else None
    cls = torch.full((w.n_tot,), 255, dtype=torch.uint8, device=dev) if want_class else None
    pl.embed_forward(g, t_feats, t_place, t_cur, wt, logits, probs, emb, pooled, out_class=cls)
    torch.cuda.synchronize()
    out = dict(logits=logits.cpu().numpy(), probs=probs.cpu().numpy(), pooled=pooled.cpu().numpy(),
               emb=None if emb is None else emb.cpu().numpy(),
               classes=None if cls is None else cls.cpu().numpy())
    if handles is None:
        g.close()
        wt.close()
    return out


def logit_errors(got, ref):
    """Error statistics of logits [B, D] against the oracle:
    row   worst over graphs of max_d|err| / (ATOL + RTOL * max_d|ref|)   (max-norm per graph)
    elem  worst over elements of |err| / (ATOL + RTOL * |ref|)           (literal, per element)
    big   the same over elements with |ref| >= 0.1 * max_d|ref| (not formed by cancellation)
    scale worst |err| / max_d|ref|
    n_elem_fail  number of elements outside the literal per-element bound"""
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, np.shape(ref)[-1])
    got = np.asarray(got, dtype=np.float64).reshape(ref.shape)
    if ref.size == 0:
        return dict(row=0.0, elem=0.0, big=0.0, scale=0.0, n_elem_fail=0)
    err = np.abs(got - ref)
    row_scale = np.max(np.abs(ref), axis=-1, keepdims=True)
    elem = err / (ATOL + RTOL * np.abs(ref))
    big = np.abs(ref) >= 0.1 * row_scale
    return dict(row=float(np.max(np.max(err, axis=-1, keepdims=True) / (ATOL + RTOL * row_scale))),
                elem=float(elem.max()), big=float(elem[big].max()),
                scale=float(np.max(err / np.maximum(row_scale, 1e-300))),
                n_elem_fail=int(np.sum(elem > 1.0)))


def assert_logits_close(got, ref, what="", max_fail_frac=0.0):
    """The bar for fp32 logits against the float64 oracle: 1e-4 relative + 1e-5 absolute.

    It is applied (a) to every graph's logit vector in the max norm, (b) literally, per
    element, to every logit that is not small against its own row (|ref| >= 0.1 max|ref|),
    and (c) literally to every other element too, except for at most `max_fail_frac` of all
    elements.  (c) is 0 unless the caller states a ceiling: with raw feature scales (output
    sizes about e^10) a logit that the last linear layer forms by cancellation (|ref| << the
    terms it sums) cannot meet a bound relative to its own size in fp32 arithmetic, its error
    is set by the row's scale; the tests on such inputs state the measured fraction as their
    ceiling, and the same graphs with features scaled to O(1) are held to the literal bound
    on every element."""
    assert np.isfinite(got).all(), f"{what}: non-finite logits"
    e = logit_errors(got, ref)
    msg = (f"{what}: row-norm ratio {e['row']:.3g}, per-element ratio {e['elem']:.3g} "
           f"({e['n_elem_fail']} of {np.size(ref)} elements outside the literal bound), "
           f"worst error {e['scale']:.3g} of the row scale")
    assert e["row"] <= 1.0 and e["big"] <= 1.0, msg
    assert e["n_elem_fail"] <= max_fail_frac * np.size(ref), msg
    return e


def row_error_ratio(got, ref, width):
    """Worst over rows of max|err| / max|ref| where a row is `width` consecutive values of the
    last axis (one direction's state of one node, one pooled vector): an error confined to one
    node or one vector is measured against that node's own scale, not the batch's."""
    ref = np.asarray(ref, dtype=np.float64).reshape(-1, width)
    got = np.asarray(got, dtype=np.float64).reshape(-1, width)
    if ref.size == 0:
        return 0.0
    scale = np.abs(ref).max(axis=1)
    err = np.abs(got - ref).max(axis=1)
    return float(np.max(err / np.maximum(scale, 1e-30) * (scale > 0) + (err > 0) * (scale == 0) * 1e30))


ROW_TOL = 2e-5      # per-row bar of embeddings and pooled sums (see assert_rows_close)


def assert_rows_close(got, ref, width, what="", tol=ROW_TOL):
    """Embeddings [N, 2H] (width H: each direction's state of each node on its own) and pooled
    sums [B, 3, G, H] (width H) against the oracle: every row within `tol` of its own largest
    entry.  fp32 arithmetic with exact products and fp32 accumulation over a few hundred terms
    of the row's scale gives errors of a few 1e-7 of that scale per layer; the bar leaves room
    for the depth of the graphs (errors add up along a path), not for a dropped term."""
    r = row_error_ratio(got, ref, width)
    assert r <= tol, f"{what}: worst row error {r:.3g} of the row's own scale (bar {tol:g})"
    return r


def normalised(w):
    """The same workload with run times and output sizes divided by their batch means, i.e.
    features of order one (the paper states no normalisation; this is the test's own input)."""
    import copy
    v = copy.copy(w)
    f = np.array(w.node_feats, dtype=np.float64, copy=True)
    f[:, 0] /= f[:, 0].mean()
    f[:, 1] /= f[:, 1].mean()
    v.node_feats = f.astype(np.float32)
    return v


def assert_probs_close(got, ref_probs, ref_logits, what=""):
    """Softmax outputs: a logit error of delta moves a probability p by at most about
    2 p delta, so the bound follows from the logit bound of the row."""
    ref_logits = np.asarray(ref_logits, dtype=np.float64)
    delta = ATOL + RTOL * np.max(np.abs(ref_logits), axis=-1, keepdims=True)
    growth = np.expm1(np.minimum(2.0 * delta, 50.0))          # vacuous once rows saturate
    bound = np.minimum(1.0, 1e-6 + np.asarray(ref_probs) * growth + 1e-6 * delta)
    assert np.all(np.abs(np.asarray(got, dtype=np.float64) - ref_probs) <= bound), what
    assert np.allclose(np.asarray(got).sum(axis=-1), 1.0, atol=1e-5), what


def custom_workload(rng, sizes, D, H, n_layers=2, k_sweeps=1, group=1, weight_dtype="fp32", p_edge=0.3,
                    w_scale=0.1):
    """A ragged batch of random DAGs with a random state and random weights."""
    from workloads import tiny_random_dag, weight_count
    from workloads.synthetic import Workload
    n_nodes, n_edges, srcs, dsts, feats, places, curs = [], [], [], [], [], [], []
    for n in sizes:
        s, d = tiny_random_dag(rng, n, p_edge)
        n_nodes.append(n); n_edges.append(len(s)); srcs.append(s); dsts.append(d)
        feats.append(np.stack([rng.lognormal(0, 1, n), rng.lognormal(2, 1, n), (rng.random(n) < 0.5)], axis=1))
        places.append(rng.integers(0, D, n)); curs.append(rng.integers(n))
    weights = rng.normal(0, w_scale, weight_count(D, H, n_layers, bool(group))).astype(np.float32)
    return Workload(name="custom", B=len(sizes), D=D, H=H, n_layers=n_layers, k_sweeps=k_sweeps,
                    group_by_device=group, weight_dtype=weight_dtype,
                    n_nodes=np.array(n_nodes, np.int32), n_edges=np.array(n_edges, np.int32),
                    edge_src=np.concatenate(srcs).astype(np.int32),
                    edge_dst=np.concatenate(dsts).astype(np.int32),
                    node_feats=np.concatenate(feats).astype(np.float32),
                    placement=np.concatenate(places).astype(np.int32),
                    cur_node=np.array(curs, np.int32), weights=weights)


def run_gradient(w, actions, coeff, handles=None, path=0, accumulate_into=None, cur_node=None,
                 entropy_coeff=None):
    """pl_policy_gradient of workload `w` on cuda:0.  Returns dict(grad, logits, logp) as numpy."""
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    if handles is None:
        g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
        wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype,
                        getattr(w, "single_set", 0))
        if path:
            wt.set_path(path)
    else:
        g, wt = handles
    t_feats = torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev)
    t_place = torch.from_numpy(np.ascontiguousarray(w.placement, dtype=np.int32)).to(dev)
    t_cur = torch.from_numpy(np.ascontiguousarray(w.cur_node if cur_node is None else cur_node, dtype=np.int32)).to(dev)
    t_act = torch.from_numpy(np.ascontiguousarray(actions, dtype=np.int32)).to(dev)
    t_coef = torch.from_numpy(np.ascontiguousarray(coeff, dtype=np.float32)).to(dev)
    n_par = pl.weights_count(w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    if accumulate_into is None:
        grad = torch.full((n_par,), float("nan"), dtype=torch.float32, device=dev)
    else:
        grad = torch.from_numpy(np.ascontiguousarray(accumulate_into, dtype=np.float32)).to(dev)
    logits = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    logp = torch.full((w.B,), 7.0, dtype=torch.float32, device=dev)
    ent = torch.full((w.B,), 7.0, dtype=torch.float32, device=dev)
    t_ent = None if entropy_coeff is None else torch.from_numpy(np.ascontiguousarray(entropy_coeff, dtype=np.float32)).to(dev)
    pl.policy_gradient(g, t_feats, t_place, t_cur, wt, t_act, t_coef, grad, logits, logp,
                       accumulate=accumulate_into is not None, entropy_coeff=t_ent,
                       out_entropy=None if entropy_coeff is None else ent)
    torch.cuda.synchronize()
    out = dict(grad=grad.cpu().numpy(), logits=logits.cpu().numpy(), logp=logp.cpu().numpy(),
               entropy=ent.cpu().numpy())
    if handles is None:
        g.close()
        wt.close()
    return out
