"""Shared helpers of the GPU parity tests: run the HIP library on a workload through the
C ABI and return numpy arrays; compare with the float64 oracle."""
import numpy as np

RTOL, ATOL = 1e-4, 1e-5     # fp32 logits vs the float64 oracle


def run_library(w, placement=None, cur_node=None, done=None, want_emb=True, handles=None, path=0):
    """One forward pass of workload `w` on cuda:0.  Returns dict of numpy arrays."""
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    if handles is None:
        g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
        wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device,
                        w.weight_dtype)
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
    pl.embed_forward(g, t_feats, t_place, t_cur, wt, logits, probs, emb, pooled)
    torch.cuda.synchronize()
    out = dict(logits=logits.cpu().numpy(), probs=probs.cpu().numpy(), pooled=pooled.cpu().numpy(),
               emb=None if emb is None else emb.cpu().numpy())
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


def assert_logits_close(got, ref, what=""):
    """The bar for fp32 logits against the float64 oracle: 1e-4 relative + 1e-5 absolute.

    It is applied (a) to every graph's logit vector in the max norm and (b) literally, per
    element, to every logit that is not small against its own row (|ref| >= 0.1 max|ref|).
    A logit that the last linear layer forms by cancellation (|ref| << the terms it sums)
    cannot meet a bound relative to its own size in fp32 arithmetic: its error is set by
    the row's scale.  Such elements are counted and reported, not hidden: `n_elem_fail`."""
    assert np.isfinite(got).all(), f"{what}: non-finite logits"
    e = logit_errors(got, ref)
    msg = (f"{what}: row-norm ratio {e['row']:.3g}, per-element ratio {e['elem']:.3g} "
           f"({e['n_elem_fail']} of {np.size(ref)} elements outside the literal bound), "
           f"worst error {e['scale']:.3g} of the row scale")
    assert e["row"] <= 1.0 and e["big"] <= 1.0, msg
    return e


def assert_probs_close(got, ref_probs, ref_logits, what=""):
    """Softmax outputs: a logit error of delta moves a probability p by at most about
    2 p delta, so the bound follows from the logit bound of the row."""
    ref_logits = np.asarray(ref_logits, dtype=np.float64)
    delta = ATOL + RTOL * np.max(np.abs(ref_logits), axis=-1, keepdims=True)
    growth = np.expm1(np.minimum(2.0 * delta, 50.0))          # vacuous once rows saturate
    bound = np.minimum(1.0, 1e-6 + np.asarray(ref_probs) * growth + 1e-6 * delta)
    assert np.all(np.abs(np.asarray(got, dtype=np.float64) - ref_probs) <= bound), what
    assert np.allclose(np.asarray(got).sum(axis=-1), 1.0, atol=1e-5), what
