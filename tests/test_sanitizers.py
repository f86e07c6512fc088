"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer: the C oracle and the
library's host-side layout and gather-plan builders are compiled with
-fsanitize=address,undefined into small executables (tests/sanitize/), run on real batches, on
the three golden examples and on inputs that take the error paths, and must (a) finish without a
sanitizer report and (b) give, bit for bit, what the ordinary builds give."""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

import oracle
from workloads import make_workload, tiny_random_dag

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")
FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-static-libasan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")

pytestmark = pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")


@pytest.fixture(scope="module")
def oracle_exe(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "oracle_san")
    subprocess.run(["gcc", "-std=c11", *FLAGS, "-fopenmp", os.path.join(ROOT, "oracle", "placeto_oracle.c"),
                    os.path.join(SAN, "oracle_driver.c"), "-o", out, "-lm"], check=True)
    return out


@pytest.fixture(scope="module")
def layout_exe(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("san") / "layout_san")
    csrc = os.path.join(ROOT, "paper_1906_08879_amd", "csrc")
    subprocess.run(["g++", "-std=c++17", *FLAGS, "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                    "-I" + os.path.join(ROOT, "include"), "-I" + csrc, os.path.join(csrc, "layout.cpp"),
                    os.path.join(csrc, "plan.cpp"), os.path.join(SAN, "layout_driver.cpp"), "-o", out], check=True)
    return out


def _run(exe, blob, tmp_path):
    src, dst = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(src, "wb") as f:
        f.write(blob)
    r = subprocess.run([exe, src, dst], capture_output=True, text=True, env=ENV, timeout=600)
    assert r.returncode == 0 and "Sanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]
    return open(dst, "rb").read()


def _oracle_blob(w, cur=None):
    blob = oracle.weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    cur = w.cur_node if cur is None else cur
    parts = [np.array([w.D, w.H, w.n_layers, w.k_sweeps, w.group_by_device, getattr(w, "single_set", 0), w.B,
                       w.n_tot, w.e_tot], np.int32), np.array([blob.size], np.int64),
             w.n_nodes.astype(np.int32), w.n_edges.astype(np.int32), w.edge_src.astype(np.int32),
             w.edge_dst.astype(np.int32), w.placement.astype(np.int32), np.asarray(cur, np.int32),
             np.asarray(w.node_feats, np.float64), np.asarray(blob, np.float64)]
    return b"".join(np.ascontiguousarray(p).tobytes() for p in parts)


def _check_oracle(w, oracle_exe, tmp_path):
    raw = _run(oracle_exe, _oracle_blob(w), tmp_path)
    G = w.D if w.group_by_device else 1
    at = 0

    def take(dtype, n):
        nonlocal at
        a = np.frombuffer(raw, dtype=dtype, count=n, offset=at)
        at += a.nbytes
        return a
    status = take(np.int32, 2 * w.B + 1)
    assert not status.any()
    td, bu, cls = take(np.int32, w.n_tot), take(np.int32, w.n_tot), take(np.uint8, w.n_tot)
    logits, probs = take(np.float64, w.B * w.D), take(np.float64, w.B * w.D)
    emb, pooled = take(np.float64, w.n_tot * 2 * w.H), take(np.float64, w.B * 3 * G * w.H)
    assert at == len(raw)
    ref = oracle.forward_workload(w, n_threads=2, want_emb=True)
    np.testing.assert_array_equal(logits, ref["logits"].ravel())
    np.testing.assert_array_equal(probs, ref["probs"].ravel())
    np.testing.assert_array_equal(emb, ref["emb"].ravel())
    np.testing.assert_array_equal(pooled, ref["pooled"].ravel())
    for b in range(w.B):
        n, src, dst, *_ = w.graph(b)
        sl = slice(int(w.node_off[b]), int(w.node_off[b + 1]))
        t, u = oracle.levels(n, src, dst)
        np.testing.assert_array_equal(td[sl], t)
        np.testing.assert_array_equal(bu[sl], u)
        np.testing.assert_array_equal(cls[sl], oracle.classes(n, src, dst, int(w.cur_node[b])))


@pytest.mark.parametrize("name,B,kw", [("random32", 1, {}), ("layered200", 3, {}),
                                        ("inception", 2, dict(k_sweeps=2, group_by_device=0, n_layers=1)),
                                        ("nasnet", 1, {})])
def test_oracle_under_sanitizers(name, B, kw, oracle_exe, tmp_path):
    _check_oracle(make_workload(name, B=B, **kw), oracle_exe, tmp_path)


class SanitizedOracle:
    """Stands where the pins expect the loaded oracle library: every call is marshalled to the
    executable built with the sanitizers and its results are copied back into the caller's arrays."""

    def __init__(self, exe, tmp_path):
        self.exe, self.tmp = exe, tmp_path
        self.real = oracle.load()

    def orc_weight_count(self, cfg):
        return self.real.orc_weight_count(cfg)            # a size formula: no memory to check

    def _call(self, cfg, n, n_edges, ps, pd, feats, placement, cur, weights):
        arr = lambda p, k, dt: np.array(np.ctypeslib.as_array(p, shape=(k,)), dtype=dt) if k else np.zeros(0, dt)
        src, dst = arr(ps, n_edges, np.int32), arr(pd, n_edges, np.int32)
        parts = [np.array([cfg.D, cfg.H, cfg.n_layers, cfg.k_sweeps, cfg.group_by_device, cfg.single_set, 1, n,
                           n_edges], np.int32), np.array([len(weights)], np.int64), np.array([n], np.int32),
                 np.array([n_edges], np.int32), src, dst, np.asarray(placement, np.int32), np.array([cur], np.int32),
                 np.asarray(feats, np.float64), np.asarray(weights, np.float64)]
        return _run(self.exe, b"".join(np.ascontiguousarray(p).tobytes() for p in parts), self.tmp)

    def orc_forward_graph(self, cfgref, n, n_edges, ps, pd, pf, pp, cur, pw, p_logits, p_probs, p_emb, p_pooled):
        cfg = cfgref._obj
        nw = int(self.real.orc_weight_count(cfgref))
        G = cfg.D if cfg.group_by_device else 1
        feats = np.ctypeslib.as_array(pf, shape=(n * 3,))
        raw = self._call(cfg, n, n_edges, ps, pd, feats, np.ctypeslib.as_array(pp, shape=(n,)), cur,
                         np.ctypeslib.as_array(pw, shape=(nw,)))
        status = np.frombuffer(raw, np.int32, 3)
        at = 12 + 8 * n + n
        for ptr, k in ((p_logits, cfg.D), (p_probs, cfg.D), (p_emb, n * 2 * cfg.H), (p_pooled, 3 * G * cfg.H)):
            np.ctypeslib.as_array(ptr, shape=(k,))[:] = np.frombuffer(raw, np.float64, k, at)
            at += 8 * k
        assert at == len(raw)
        return int(status[2])

    def orc_classes(self, n, n_edges, ps, pd, cur, p_cls):
        cfg = oracle.OracleCfg(1, 1, 1, 0, 1, 0)
        raw = self._call(cfg, n, n_edges, ps, pd, np.zeros(3 * n), np.zeros(n, np.int32), cur, np.zeros(0))
        np.ctypeslib.as_array(p_cls, shape=(n,))[:] = np.frombuffer(raw, np.uint8, n, 12 + 8 * n)
        return int(np.frombuffer(raw, np.int32, 3)[1])


def test_oracle_pins_under_sanitizers(oracle_exe, tmp_path):
    """Three pins of the oracle, run as they are against the sanitized build: the hand-derived
    asymmetric two-node example, the three-node chain and the diamond (tests/golden/)."""
    import oracle_pins
    lib = SanitizedOracle(oracle_exe, tmp_path)
    oracle_pins.pin_two_node_asymmetric(lib)
    oracle_pins.pin_chain3(lib)
    oracle_pins.pin_diamond(lib)


def test_oracle_error_paths_under_sanitizers(oracle_exe, tmp_path):
    """A cyclic graph and an out-of-range edge: the error returns free what they allocated."""
    w = make_workload("random32")
    bad = make_workload("random32")
    bad.edge_src = np.concatenate([w.edge_src, w.edge_dst[:1]]).astype(np.int32)     # closes a cycle
    bad.edge_dst = np.concatenate([w.edge_dst, w.edge_src[:1]]).astype(np.int32)
    bad.n_edges = (w.n_edges + 1).astype(np.int32)
    bad.__post_init__()
    raw = _run(oracle_exe, _oracle_blob(bad), tmp_path)
    status = np.frombuffer(raw, dtype=np.int32, count=3)
    assert status[0] != 0 and status[2] != 0          # levels and the forward pass refuse a cycle


def _layout_blob(n_nodes, n_edges, src, dst):
    parts = [np.array([len(n_nodes), len(src)], np.int32), np.asarray(n_nodes, np.int32), np.asarray(n_edges, np.int32),
             np.asarray(src, np.int32), np.asarray(dst, np.int32)]
    return b"".join(np.ascontiguousarray(p).tobytes() for p in parts)


def _check_layout(w, layout_exe, tmp_path):
    import paper_1906_08879_amd as pl
    raw = _run(layout_exe, _layout_blob(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst), tmp_path)
    status, = struct.unpack_from("<i", raw, 0)
    assert status == 0
    n_tot, e_tot, depth = struct.unpack_from("<qqi", raw, 4)
    assert (n_tot, e_tot) == (w.n_tot, w.e_tot)
    at = 4 + 20

    def take(dtype, n):
        nonlocal at
        a = np.frombuffer(raw, dtype=dtype, count=n, offset=at)
        at += a.nbytes
        return a
    td, bu, td_o, bu_o = (take(np.int32, n_tot) for _ in range(4))
    par_ptr, chi_ptr = take(np.int64, n_tot + 1), take(np.int64, n_tot + 1)
    par_idx, chi_idx = take(np.int32, e_tot), take(np.int32, e_tot)
    g = pl.GraphBatch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst)        # the ordinary build, host calls only
    assert depth == g.max_depth
    lt, lb = g.levels()
    lay = g.layout()
    np.testing.assert_array_equal(td, lt)
    np.testing.assert_array_equal(bu, lb)
    for name, arr in (("td_order", td_o), ("bu_order", bu_o), ("par_ptr", par_ptr), ("chi_ptr", chi_ptr),
                      ("par_idx", par_idx), ("chi_idx", chi_idx)):
        np.testing.assert_array_equal(arr, lay[name], err_msg=name)
    g.close()
    for dirn in range(2):                                                  # the sweep kernel's gather plan
        n_ck, n_rec, n_ovf = take(np.int64, 3)
        ck_off, rec, ovf = take(np.int32, int(n_ck)), take(np.uint32, int(n_rec)), take(np.int32, int(n_ovf))
        _check_plan(w, dirn, td if dirn == 0 else bu, td_o if dirn == 0 else bu_o, ck_off, rec.reshape(-1, 8, 4), ovf)
    assert at == len(raw)
    for b in range(w.B):                                                   # and the oracle's levels
        n, src, dst, *_ = w.graph(b)
        t, u = oracle.levels(n, src, dst)
        sl = slice(int(w.node_off[b]), int(w.node_off[b + 1]))
        np.testing.assert_array_equal(td[sl], t)
        np.testing.assert_array_equal(bu[sl], u)


RING, CH, MAX_NEAR = 4, 8, 5      # constants of the plan (sweep_plan.h)


def _check_plan(w, dirn, level, order, ck_off, rec, ovf):
    """Every row record of the gather plan against the edge list: the chunk cuts levels in bucket
    order; the near slots (messages of the last RING chunks), the far source or the row's list name
    exactly the row's neighbours; the chunk-wide bits say what the rows need."""
    assert len(ck_off) == w.B + 1
    for b in range(w.B):
        n0, n = int(w.node_off[b]), int(w.n_nodes[b])
        e0, e1 = int(w.edge_off[b]), int(w.edge_off[b + 1])
        src, dst = w.edge_src[e0:e1], w.edge_dst[e0:e1]
        nbr = [[] for _ in range(n)]
        for u, v in zip(src.tolist(), dst.tolist()):
            (nbr[v] if dirn == 0 else nbr[u]).append(u if dirn == 0 else v)
        lev, ordr = level[n0:n0 + n], order[n0:n0 + n]
        chunk_of, row_of = np.full(n, -1), np.full(n, -1)
        pos = 0
        recs = rec[ck_off[b]:ck_off[b + 1]]
        for c, ck in enumerate(recs):
            info = int(ck[0, 3])
            rows = ((info >> 24) & 7) + 1
            assert all(int(ck[r, 3]) >> 24 == info >> 24 for r in range(CH))          # chunk-wide bits agree
            assert all(int(ck[r, 2]) == pos for r in range(CH))                       # first bucket position
            ids = [int(ck[r, 3]) & 0xFFFFFF for r in range(CH)]
            assert ids[:rows] == ordr[pos:pos + rows].tolist() and all(i == 0xFFFFFF for i in ids[rows:])
            assert len(set(lev[ids[:rows]].tolist())) == 1                            # one level per chunk
            if pos + rows < n and rows < CH:
                assert lev[ordr[pos + rows]] != lev[ids[0]]                           # a chunk ends with its level or when full
            any_listed = any_far = False
            widest = 0
            for r in range(rows):
                v = ids[r]
                chunk_of[v], row_of[v] = c, r
                w0, w1 = int(ck[r, 0]), int(ck[r, 1])
                got = []
                if w0 & (1 << 30):
                    any_listed = True
                    cnt = w0 & 0xFFFFFF
                    for x in ovf[w1:w1 + cnt].tolist():
                        if x >= 0:
                            assert c - chunk_of[x] > RING
                            got.append(x)
                        else:
                            slot = -1 - x
                            u = [q for q in nbr[v] if chunk_of[q] % RING == slot // CH and row_of[q] == slot % CH
                                 and 0 < c - chunk_of[q] <= RING]
                            assert len(u) == 1
                            got.append(u[0])
                    near = sum(1 for q in nbr[v] if c - chunk_of[q] <= RING)
                    assert near > MAX_NEAR or len(nbr[v]) - near > 1                  # listed only when needed
                else:
                    k_near = 0
                    for k in range(MAX_NEAR):
                        slot = (w0 >> (6 * k)) & 63
                        if slot == RING * CH:
                            continue
                        assert slot < RING * CH and k == k_near                        # used slots first
                        k_near += 1
                        u = [q for q in nbr[v] if chunk_of[q] % RING == slot // CH and row_of[q] == slot % CH
                             and 0 < c - chunk_of[q] <= RING]
                        assert len(u) == 1
                        got.append(u[0])
                    widest = max(widest, k_near)
                    if w1 != 0xFFFFFFFF:
                        any_far = True
                        assert c - chunk_of[w1] > RING
                        got.append(w1)
                assert sorted(got) == sorted(nbr[v]), (b, c, r)
            for r in range(rows, CH):
                assert int(ck[r, 0]) == sum((RING * CH) << (6 * k) for k in range(MAX_NEAR)) and int(ck[r, 1]) == 0xFFFFFFFF
            assert (info >> 27) & 1 == int(any_listed) and (info >> 28) & 1 == int(any_far)
            assert (info >> 29) & 3 == (0 if widest <= 1 else (1 if widest == 2 else 2))
            pos += rows
        assert pos == n


@pytest.mark.parametrize("name,B", [("random32", 1), ("layered200", 6), ("nmt", 2), ("nasnet", 2)])
def test_layout_and_plan_builders_under_sanitizers(name, B, layout_exe, tmp_path):
    _check_layout(make_workload(name, B=B), layout_exe, tmp_path)


def test_layout_builder_on_dense_and_degenerate_graphs_under_sanitizers(layout_exe, tmp_path):
    """Dense DAGs (rows that overflow their plan records, many far sources), single nodes,
    edgeless graphs, an empty batch, and every refusal (self loop, repeated edge, cycle, bad id)."""
    from workloads.synthetic import Workload
    rng = np.random.default_rng(5)
    sizes = [150, 1, 40, 2, 90]
    srcs, dsts = zip(*[tiny_random_dag(rng, n, p) for n, p in zip(sizes, (0.5, 0.0, 0.0, 1.0, 0.2))])
    w = Workload(name="dense", B=len(sizes), D=2, H=8, n_layers=2, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 n_nodes=np.array(sizes, np.int32), n_edges=np.array([len(s) for s in srcs], np.int32),
                 edge_src=np.concatenate(srcs).astype(np.int32), edge_dst=np.concatenate(dsts).astype(np.int32),
                 node_feats=np.zeros((sum(sizes), 3), np.float32), placement=np.zeros(sum(sizes), np.int32),
                 cur_node=np.zeros(len(sizes), np.int32), weights=np.zeros(1, np.float32))
    _check_layout(w, layout_exe, tmp_path)
    raw = _run(layout_exe, _layout_blob([], [], [], []), tmp_path)
    assert struct.unpack_from("<i", raw, 0)[0] == 0
    for src, dst, code in (([0, 1], [1, 1], -4), ([0, 0], [1, 1], -5), ([0, 1, 2], [1, 2, 0], -6), ([0, 5], [1, 2], -3)):
        raw = _run(layout_exe, _layout_blob([3], [len(src)], src, dst), tmp_path)
        assert struct.unpack_from("<i", raw, 0)[0] == code
