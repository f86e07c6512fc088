"""Float64 CPU oracle for the Placeto policy forward pass (Section 2.2, Appendix A.7).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the benchmark's
cpu_baseline leg.  It shares no code with the HIP library and never imports it.

`build()` compiles oracle/placeto_oracle.c with gcc; the functions below marshal numpy
arrays into it.  The only arithmetic on the Python side is the rounding of weight matrices
to bfloat16 (round-to-nearest-even) for the configuration that stores its weights in that
format; the oracle then uses those rounded values exactly, in float64, with unrounded
activations.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "placeto_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


class OracleCfg(ctypes.Structure):
    _fields_ = [("D", ctypes.c_int32), ("H", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("k_sweeps", ctypes.c_int32), ("group_by_device", ctypes.c_int32),
                ("single_set", ctypes.c_int32)]


def build(force: bool = True, src: str = _SRC, out: str = _LIB) -> str:
    """Compile the C oracle (plain gcc, no fast-math so summation order is as written)."""
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        cmd = ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-fopenmp", "-shared", "-fPIC",
               "-o", out, src, "-lm"]
        subprocess.run(cmd, check=True)
    return out


def load(path: Optional[str] = None):
    """Load a compiled oracle library and declare its signatures."""
    lib = ctypes.CDLL(path or build(force=False))
    i32p = ctypes.POINTER(ctypes.c_int32)
    f64p = ctypes.POINTER(ctypes.c_double)
    u8p = ctypes.POINTER(ctypes.c_uint8)
    cfgp = ctypes.POINTER(OracleCfg)
    lib.orc_weight_count.restype = ctypes.c_size_t
    lib.orc_weight_count.argtypes = [cfgp]
    lib.orc_levels.restype = ctypes.c_int
    lib.orc_levels.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, i32p, i32p]
    lib.orc_classes.restype = ctypes.c_int
    lib.orc_classes.argtypes = [ctypes.c_int32, ctypes.c_int32, i32p, i32p, ctypes.c_int32, u8p]
    lib.orc_forward_graph.restype = ctypes.c_int
    lib.orc_forward_graph.argtypes = [cfgp, ctypes.c_int32, ctypes.c_int32, i32p, i32p, f64p,
                                      i32p, ctypes.c_int32, f64p, f64p, f64p, f64p, f64p]
    lib.orc_forward_batch.restype = ctypes.c_int
    lib.orc_forward_batch.argtypes = [cfgp, ctypes.c_int32, i32p, i32p, i32p, i32p, f64p, i32p,
                                      i32p, f64p, f64p, f64p, f64p, f64p, ctypes.c_int32]
    return lib


def _get():
    global _lib
    if _lib is None:
        _lib = load()
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _out(shape):
    a = np.zeros(shape, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 values rounded to the nearest bfloat16 (ties to even), returned as float32."""
    bits = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return rounded.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def weights_as_stored(weights: np.ndarray, D: int, H: int, n_layers: int,
                      group_by_device: int, weight_dtype: str) -> np.ndarray:
    """The float64 blob the oracle computes with.  For 'bf16' every weight matrix is
    rounded to bfloat16; biases stay float32."""
    w = np.array(weights, dtype=np.float32, copy=True)
    if weight_dtype == "bf16":
        F, G = D + 4, (D if group_by_device else 1)
        shapes = [(F, H)]
        shapes += [(H, H)] * (4 * n_layers)
        for _ in range(3):
            shapes += [(2 * H, H)] + [(H, H)] * (n_layers - 1)
        shapes += [(H, H)] * (3 * n_layers)
        shapes += [((2 + 3 * G) * H, H), (H, D)]
        pos = 0
        for n_in, n_out in shapes:
            w[pos:pos + n_in * n_out] = round_to_bf16(w[pos:pos + n_in * n_out])
            pos += n_in * n_out + n_out
        assert pos == w.size
    elif weight_dtype != "fp32":
        raise ValueError(weight_dtype)
    return w.astype(np.float64)


def weight_count(D, H, n_layers=2, group_by_device=1) -> int:
    cfg = OracleCfg(D, H, n_layers, 1, group_by_device)
    return int(_get().orc_weight_count(ctypes.byref(cfg)))


def levels(n, src, dst, lib=None):
    """Longest-path levels from the roots (top-down) and from the leaves (bottom-up)."""
    src, ps = _i32(src)
    dst, pd = _i32(dst)
    td = np.zeros(n, dtype=np.int32)
    bu = np.zeros(n, dtype=np.int32)
    rc = (lib or _get()).orc_levels(n, len(src), ps, pd, td.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                           bu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc:
        raise ValueError(f"orc_levels failed: {rc}")
    return td, bu


def level_order(level: np.ndarray) -> np.ndarray:
    """Nodes sorted by (level, node id): the bucket order of the layout."""
    return np.lexsort((np.arange(len(level)), level)).astype(np.int32)


def classes(n, src, dst, cur, lib=None) -> np.ndarray:
    """0 = current node, 1 = S_parents, 2 = S_children, 3 = S_parallel (Section 2.2 step 3)."""
    src, ps = _i32(src)
    dst, pd = _i32(dst)
    cls = np.zeros(n, dtype=np.uint8)
    rc = (lib or _get()).orc_classes(n, len(src), ps, pd, int(cur),
                            cls.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)))
    if rc:
        raise ValueError(f"orc_classes failed: {rc}")
    return cls


def forward_graph(n, src, dst, feats, placement, cur, weights, D, H, n_layers=2, k_sweeps=1,
                  group_by_device=1, lib=None, single_set=0):
    """One graph.  Returns dict(logits [D], probs [D], emb [n,2H], pooled [3,G,H])."""
    lib = lib or _get()
    cfg = OracleCfg(D, H, n_layers, k_sweeps, group_by_device, single_set)
    G = D if group_by_device else 1
    src, ps = _i32(src)
    dst, pd = _i32(dst)
    feats, pf = _f64(np.asarray(feats).reshape(n, 3))
    placement, pp = _i32(placement)
    weights, pw = _f64(weights)
    if weights.size != lib.orc_weight_count(ctypes.byref(cfg)):
        raise ValueError("weight blob has the wrong size")
    logits, pl = _out(D)
    probs, pr = _out(D)
    emb, pe = _out((n, 2 * H))
    pooled, pq = _out((3, G, H))
    rc = lib.orc_forward_graph(ctypes.byref(cfg), n, len(src), ps, pd, pf, pp, int(cur), pw,
                               pl, pr, pe, pq)
    if rc:
        raise ValueError(f"orc_forward_graph failed: {rc}")
    return dict(logits=logits, probs=probs, emb=emb, pooled=pooled)


def forward_batch(n_nodes, n_edges, src, dst, feats, placement, cur, weights, D, H,
                  n_layers=2, k_sweeps=1, group_by_device=1, n_threads=1, want_emb=True,
                  lib=None, single_set=0):
    """A concatenated batch.  Returns dict(logits [B,D], probs [B,D], emb [N_tot,2H] or None,
    pooled [B,3,G,H])."""
    lib = lib or _get()
    cfg = OracleCfg(D, H, n_layers, k_sweeps, group_by_device, single_set)
    G = D if group_by_device else 1
    n_nodes, pn = _i32(n_nodes)
    n_edges, pe_ = _i32(n_edges)
    B = len(n_nodes)
    n_tot = int(n_nodes.sum())
    src, ps = _i32(src)
    dst, pd = _i32(dst)
    feats, pf = _f64(np.asarray(feats).reshape(n_tot, 3))
    placement, pp = _i32(placement)
    cur, pc = _i32(cur)
    weights, pw = _f64(weights)
    if weights.size != lib.orc_weight_count(ctypes.byref(cfg)):
        raise ValueError("weight blob has the wrong size")
    logits, pl = _out((B, D))
    probs, pr = _out((B, D))
    pooled, pq = _out((B, 3, G, H))
    if want_emb:
        emb, pe = _out((n_tot, 2 * H))
    else:
        emb, pe = None, None
    rc = lib.orc_forward_batch(ctypes.byref(cfg), B, pn, pe_, ps, pd, pf, pp, pc, pw, pl, pr, pe,
                               pq, int(n_threads))
    if rc:
        raise ValueError(f"orc_forward_batch failed: {rc}")
    return dict(logits=logits, probs=probs, emb=emb, pooled=pooled)


def forward_workload(w, n_threads=1, want_emb=True, placement=None, cur_node=None, done=None):
    """Run the oracle on a workloads.Workload (optionally with another state)."""
    feats = np.array(w.node_feats, dtype=np.float64, copy=True)
    if done is not None:
        feats[:, 2] = done
    blob = weights_as_stored(w.weights, w.D, w.H, w.n_layers, w.group_by_device, w.weight_dtype)
    return forward_batch(w.n_nodes, w.n_edges, w.edge_src, w.edge_dst, feats,
                         w.placement if placement is None else placement,
                         w.cur_node if cur_node is None else cur_node, blob, w.D, w.H,
                         w.n_layers, w.k_sweeps, w.group_by_device, n_threads, want_emb,
                         single_set=getattr(w, "single_set", 0))
