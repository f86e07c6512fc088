"""Host-side checks of the C-ABI library that need no GPU: every declared symbol is
exported, the layout builder is bit-exact against the oracle's levels and plain numpy
sorting, and malformed graphs are refused with the documented codes."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_1906_08879_amd as pl
from workloads import CONFIG_NAMES, make_workload, tiny_random_dag, weight_count

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pl.library_path()):
        from paper_1906_08879_amd.build import build
        build()
    return pl.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "placeto.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(pl_[a-z_]+)\s*\(", header))
    assert {"pl_embed_forward", "pl_graph_batch_create", "pl_weights_create"} <= names
    raw = ctypes.CDLL(pl.library_path())
    for name in sorted(names):
        assert hasattr(raw, name), f"{name} is declared but not exported"
    assert b"gfx950" in lib.pl_version()


def test_weight_count_agrees_with_interface(lib):
    for D, H, L, g in [(2, 8, 2, 1), (4, 32, 2, 1), (8, 128, 2, 1), (3, 5, 1, 0), (4, 64, 3, 0)]:
        assert pl.weights_count(D, H, L, 1, g) == weight_count(D, H, L, bool(g))
    assert pl.weights_count(0, 8) == 0 and pl.weights_count(4, 257) == 0


def _check_layout(w):
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)
    td, bu = g.levels()
    lay = g.layout()
    assert g.B == w.B and g.n_tot == w.n_tot and g.e_tot == w.e_tot
    depth = 0
    for b in range(w.B):
        n, src, dst, *_ = w.graph(b)
        n0, n1 = w.node_off[b], w.node_off[b + 1]
        otd, obu = oracle.levels(n, src, dst)
        np.testing.assert_array_equal(td[n0:n1], otd)
        np.testing.assert_array_equal(bu[n0:n1], obu)
        np.testing.assert_array_equal(lay["td_order"][n0:n1], oracle.level_order(otd))
        np.testing.assert_array_equal(lay["bu_order"][n0:n1], oracle.level_order(obu))
        depth = max(depth, int(otd.max()) + 1)
        # CSR: parents of v ascending = sorted sources of edges into v (plain numpy)
        for ptr, idx, key, val in ((lay["par_ptr"], lay["par_idx"], dst, src),
                                   (lay["chi_ptr"], lay["chi_idx"], src, dst)):
            o = np.lexsort((val, key))
            np.testing.assert_array_equal(idx[ptr[n0]:ptr[n1]], val[o])
            np.testing.assert_array_equal(np.diff(ptr[n0:n1 + 1]), np.bincount(key, minlength=n))
    assert g.max_depth == depth
    g.close()


@pytest.mark.parametrize("name", CONFIG_NAMES)
def test_layout_bit_exact_on_workloads(lib, name):
    _check_layout(make_workload(name, B=3 if name != "random32" else 1))


def test_layout_on_tiny_and_ragged_batches(lib):
    rng = np.random.default_rng(3)
    n_nodes, n_edges, srcs, dsts = [], [], [], []
    for n in (1, 1, 2, 7, 33, 1, 64):
        s, d = tiny_random_dag(rng, n, 0.3)
        n_nodes.append(n); n_edges.append(len(s)); srcs.append(s); dsts.append(d)
    class W:  # minimal stand-in with the fields _check_layout reads
        pass
    w = W()
    w.B = len(n_nodes)
    w.n_nodes, w.n_edges = np.array(n_nodes, np.int32), np.array(n_edges, np.int32)
    w.edge_src, w.edge_dst = np.concatenate(srcs), np.concatenate(dsts)
    w.node_off = np.concatenate([[0], np.cumsum(n_nodes)])
    w.edge_off = np.concatenate([[0], np.cumsum(n_edges)])
    w.n_tot, w.e_tot = int(w.node_off[-1]), int(w.edge_off[-1])
    w.graph = lambda b: (n_nodes[b], srcs[b], dsts[b])
    _check_layout(w)


def test_empty_batch(lib):
    g = pl.GraphBatch([], [], [], [])
    assert (g.B, g.n_tot, g.e_tot, g.max_depth) == (0, 0, 0, 0)
    g.close()


@pytest.mark.parametrize("n,src,dst,code", [
    (2, [0, 1], [1, 0], -6),           # cycle
    (3, [0, 1, 2], [1, 2, 0], -6),     # longer cycle
    (2, [0], [0], -4),                 # self loop
    (2, [0, 0], [1, 1], -5),           # repeated edge
    (2, [0], [2], -3),                 # endpoint out of range
    (2, [-1], [1], -3),
    (0, [], [], -2),                   # a graph needs at least one node
])
def test_malformed_graphs_are_refused(lib, n, src, dst, code):
    with pytest.raises(pl.PlacetoError) as err:
        pl.GraphBatch([n], [len(src)], src, dst)
    assert f"({code})" in str(err.value)


def test_null_and_shape_errors(lib):
    out = ctypes.c_void_p()
    assert lib.pl_graph_batch_create(1, None, None, None, None, ctypes.byref(out)) == -1
    assert lib.pl_graph_batch_create(-1, None, None, None, None, ctypes.byref(out)) == -2
    assert lib.pl_graph_batch_levels(None, None, None) == -1
    assert lib.pl_embed_forward(None, None, None, None, None, None, None) == -1
    cfg = pl.ModelCfg(4, 32, 2, 1, 1, 0)
    blob = np.zeros(10, np.float32)
    assert lib.pl_weights_create(ctypes.byref(cfg), blob.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                 10, ctypes.byref(out)) == -2
    assert b"expected" in lib.pl_last_error()
    assert lib.pl_weights_count(ctypes.byref(pl.ModelCfg(4, 32, 2, 1, 1, 0, 1))) == \
        lib.pl_weights_count(ctypes.byref(pl.ModelCfg(4, 32, 2, 1, 1, 0, 0))) > 0
    assert lib.pl_weights_count(ctypes.byref(pl.ModelCfg(4, 32, 2, 1, 1, 0, 2))) == 0   # single_set is 0 or 1
    assert lib.pl_graph_batch_destroy(None) == 0 and lib.pl_weights_destroy(None) == 0


def test_episode_entry_points_reject_bad_arguments(lib):
    """Error paths of the MDP transition calls that need no device: NULL handles and
    impossible sizes come back as error codes, with a message."""
    import ctypes
    raw = ctypes.CDLL(pl.library_path())
    null = ctypes.c_void_p(None)
    args_step = [null, ctypes.c_int32(4), null, null, null, ctypes.c_int32(0), null, null, null, null, null, null]
    assert raw.pl_episode_step(*args_step) == -1                       # PL_ERR_NULL
    g = pl.GraphBatch([2], [1], [0], [1])
    args_step[0] = g._h
    args_step[1] = ctypes.c_int32(99)
    assert raw.pl_episode_step(*args_step) != 0                         # D out of range
    args_step[1] = ctypes.c_int32(4)
    args_step[5] = ctypes.c_int32(-1)
    assert raw.pl_episode_step(*args_step) != 0                         # negative step
    args_run = [g._h, null, null, null, null, null, null, ctypes.c_int32(0), ctypes.c_int32(1), null,
                ctypes.c_int32(0), null, null, null]
    assert raw.pl_episode_run(*args_run) == -1                          # weights handle is NULL
    raw.pl_last_error.restype = ctypes.c_char_p
    assert b"NULL" in raw.pl_last_error()
    g.close()


def test_policy_gradient_rejects_null_handles(lib):
    """pl_policy_gradient without a graph batch or weights handle returns PL_ERR_NULL with a message
    (no device is touched)."""
    import ctypes
    raw = ctypes.CDLL(pl.library_path())
    null = ctypes.c_void_p(None)
    g = pl.GraphBatch([3], [2], [0, 1], [1, 2])
    args = [g._h, null, null, null, null, null, null, ctypes.c_int32(0), null, null, null, null]
    assert raw.pl_policy_gradient(*args) == -1                          # weights handle is NULL
    args[0] = null
    assert raw.pl_policy_gradient(*args) == -1                          # graph batch is NULL
    raw.pl_last_error.restype = ctypes.c_char_p
    assert b"NULL" in raw.pl_last_error()
    g.close()


def test_reinforce_entry_points_reject_bad_arguments(lib):
    """Error paths that need no device: negative sizes, missing arrays, NULL handles."""
    import ctypes
    raw = ctypes.CDLL(pl.library_path())
    null = ctypes.c_void_p(None)
    i32 = ctypes.c_int32
    assert raw.pl_reinforce_coeff(i32(-1), i32(4), null, null, i32(0), null, null, null) == -2   # PL_ERR_SHAPE
    assert raw.pl_reinforce_coeff(i32(0), i32(4), null, null, i32(0), null, null, null) == 0     # nothing to do
    assert raw.pl_reinforce_coeff(i32(3), i32(4), null, null, i32(0), null, null, null) == -1    # PL_ERR_NULL
    g = pl.GraphBatch([2], [1], [0], [1])
    args = [g._h, null, null, null, null, null, null, null, null, i32(0), i32(1), i32(0), null, null, null, null]
    assert raw.pl_episode_gradient(*args) == -1                                                 # weights handle is NULL
    g.close()


def test_simulate_reward_rejects_bad_arguments(lib):
    import ctypes
    raw = ctypes.CDLL(pl.library_path())
    null = ctypes.c_void_p(None)
    f = ctypes.c_float
    raw.pl_simulate_reward.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, f, f, f,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                       ctypes.c_void_p]
    assert raw.pl_simulate_reward(null, 4, null, null, f(1.0), f(1.0), f(2.0), null, null, null, null, null) == -1
    g = pl.GraphBatch([2], [1], [0], [1])
    assert raw.pl_simulate_reward(g._h, 99, null, null, f(1.0), f(1.0), f(2.0), null, null, null, null, null) == -2
    assert raw.pl_simulate_reward(g._h, 4, null, null, f(-1.0), f(1.0), f(2.0), null, null, null, null, null) == -2
    assert raw.pl_simulate_reward(g._h, 4, null, null, f(1.0), f(1.0), f(-2.0), null, null, null, null, null) == -2
    assert raw.pl_simulate_reward(g._h, 4, null, null, f(1.0), f(1.0), f(2.0), null, null, null, null, null) == -1
    g.close()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: a larger --gpus ends with a message, before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                       text=True, timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_replicated_batch_has_the_layout_of_the_repeated_graph():
    """pl_graph_batch_create_replicated (R rollouts of one graph, the batch shape of the appendix's
    REINFORCE section): levels, CSR and bucket orders equal those of the graph repeated R times."""
    import paper_1906_08879_amd as pl
    from workloads import make_workload
    w = make_workload("inception", B=1)
    R = 5
    rep = pl.GraphBatch(int(w.n_nodes[0]), int(w.n_edges[0]), w.edge_src, w.edge_dst, replicate=R)
    ordinary = pl.GraphBatch(np.tile(w.n_nodes, R), np.tile(w.n_edges, R), np.tile(w.edge_src, R), np.tile(w.edge_dst, R))
    assert (rep.B, rep.n_tot, rep.e_tot, rep.max_depth) == (ordinary.B, ordinary.n_tot, ordinary.e_tot, ordinary.max_depth)
    for a, b in zip(rep.levels(), ordinary.levels()):
        np.testing.assert_array_equal(a, b)
    la, lb = rep.layout(), ordinary.layout()
    for key in la:
        np.testing.assert_array_equal(la[key], lb[key], err_msg=key)
    rep.close(); ordinary.close()
    with pytest.raises(pl.PlacetoError):
        pl.GraphBatch(3, 3, [0, 1, 2], [1, 2, 0], replicate=4)       # a cycle is refused as usual
    with pytest.raises(pl.PlacetoError):
        pl.GraphBatch(3, 1, [0], [1], replicate=0)
