"""pl_embed_forward_static, the forward pass for callers that cannot allocate: called through
the C ABI, its logits and probabilities must equal pl_embed_forward's bit for bit (same kernels,
same summation orders; only the home of the intermediate buffers differs), on two calls in a row
of which the second has the smaller input, so that what the first call left in the shared block
cannot leak into the second."""
import numpy as np
import pytest

from workloads import make_workload

pytestmark = pytest.mark.gpu


def _state(w, dev):
    import torch
    return (torch.from_numpy(np.ascontiguousarray(w.node_feats, dtype=np.float32)).to(dev),
            torch.from_numpy(np.ascontiguousarray(w.placement, dtype=np.int32)).to(dev),
            torch.from_numpy(np.ascontiguousarray(w.cur_node, dtype=np.int32)).to(dev))


def _handles(w):
    import paper_1906_08879_amd as pl
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    wt = pl.Weights(w.weights, w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, w.weight_dtype)
    return g, wt


def _reference(w, dev):
    """pl_embed_forward on fresh handles."""
    import torch
    import paper_1906_08879_amd as pl
    g, wt = _handles(w)
    f, p, c = _state(w, dev)
    logits = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    probs = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    pl.embed_forward(g, f, p, c, wt, logits, probs)
    torch.cuda.synchronize()
    out = logits.cpu().numpy(), probs.cpu().numpy()
    g.close(); wt.close()
    return out


def _static(w, dev, g=None, wt=None):
    import torch
    import paper_1906_08879_amd as pl
    own = g is None
    if own:
        g, wt = _handles(w)
        pl.graph_batch_upload(g)
    f, p, c = _state(w, dev)
    logits = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    probs = torch.full((w.B, w.D), float("nan"), dtype=torch.float32, device=dev)
    pl.embed_forward_static(g, f, p, c, wt, logits, probs)
    torch.cuda.synchronize()
    out = logits.cpu().numpy(), probs.cpu().numpy()
    if own:
        g.close(); wt.close()
    return out


def test_static_forward_equals_the_allocating_one_on_two_calls_in_a_row():
    import torch
    dev = torch.device("cuda:0")
    # matrix-core kernels (H = 128, bf16 weights, deep graphs), then a smaller batch on other
    # shapes (H = 32, fp32), then the generic kernels' shapes (H = 8) smaller still
    seq = [make_workload("nasnet", B=2), make_workload("layered200", B=5), make_workload("random32")]
    want = [_reference(w, dev) for w in seq]
    for w, (ref_logits, ref_probs) in zip(seq, want):
        print(f"[static] {w.name} B={w.B}", flush=True)
        logits, probs = _static(w, dev)
        np.testing.assert_array_equal(logits, ref_logits, err_msg=w.name)
        np.testing.assert_array_equal(probs, ref_probs, err_msg=w.name)
    # and back to the larger one: the block now holds the smaller calls' leftovers
    logits, probs = _static(seq[0], dev)
    np.testing.assert_array_equal(logits, want[0][0])


def test_static_forward_on_a_stream_of_states_and_variants():
    """Several states through one pair of handles; two sweeps and per-set pooling."""
    import torch
    import paper_1906_08879_amd as pl
    from workloads import make_states
    dev = torch.device("cuda:0")
    w = make_workload("inception", B=4, k_sweeps=2, group_by_device=0)
    placement, cur, done = make_states(w, 3)
    g, wt = _handles(w)
    pl.graph_batch_upload(g)
    g2, wt2 = _handles(w)
    for s in range(3):
        f = np.array(w.node_feats, dtype=np.float32)
        f[:, 2] = done[s]
        tf, tp, tc = (torch.from_numpy(f).to(dev), torch.from_numpy(placement[s]).to(dev),
                      torch.from_numpy(cur[s]).to(dev))
        a = torch.empty((w.B, w.D), dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        pl.embed_forward_static(g, tf, tp, tc, wt, a)
        pl.embed_forward(g2, tf, tp, tc, wt2, b)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(a.cpu().numpy(), b.cpu().numpy())
    for h in (g, wt, g2, wt2):
        h.close()


def test_static_forward_refuses_what_it_cannot_serve():
    import torch
    import paper_1906_08879_amd as pl
    dev = torch.device("cuda:0")
    w = make_workload("layered200", B=2)
    g, wt = _handles(w)
    f, p, c = _state(w, dev)
    out = torch.zeros((w.B, w.D), dtype=torch.float32, device=dev)
    with pytest.raises(pl.PlacetoError, match="pl_graph_batch_upload"):      # not on the device yet
        pl.embed_forward_static(g, f, p, c, wt, out)
    g.close(); wt.close()
    big = make_workload("nasnet", B=12)                                      # ~ 116 MB of buffers
    g, wt = _handles(big)
    pl.graph_batch_upload(g)
    assert pl.embed_forward_static_bytes(g, wt) > pl.embed_forward_static_limit()
    f, p, c = _state(big, dev)
    out = torch.zeros((big.B, big.D), dtype=torch.float32, device=dev)
    with pytest.raises(pl.PlacetoError, match="more than the fixed block"):
        pl.embed_forward_static(g, f, p, c, wt, out)
    torch.cuda.synchronize()
    assert not out.any()                                                     # nothing was launched
    g.close(); wt.close()
