"""ctypes binding with the same names as include/placeto.h: argument marshalling only.

Device buffers are torch tensors (PyTorch is used for device memory and streams, nothing
else); host arrays are numpy.  There is no fallback: if the shared library is missing or a
call fails, PlacetoError is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libplaceto.so")
_lib = None

PL_WEIGHTS = {"fp32": 0, "bf16": 1}
STAGES = ("project", "sweep", "pool", "head", "bw_head", "bw_pool", "bw_acts", "bw_chain", "bw_proj", "bw_wgrad")


class PlacetoError(RuntimeError):
    pass


class ModelCfg(ctypes.Structure):
    _fields_ = [("D", ctypes.c_int32), ("H", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("k_sweeps", ctypes.c_int32), ("group_by_device", ctypes.c_int32),
                ("weight_dtype", ctypes.c_int32), ("single_set", ctypes.c_int32)]


def library_path() -> str:
    return _LIB_PATH


def load_library(path: Optional[str] = None):
    """Load libplaceto.so and declare every signature of include/placeto.h."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or _LIB_PATH
    if not os.path.exists(path):
        raise PlacetoError(f"{path} is not built; run `python -m paper_1906_08879_amd.build` "
                           "(there is no CPU fallback)")
    lib = ctypes.CDLL(path)
    vp, i32p, i64p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
    cfgp = ctypes.POINTER(ModelCfg)
    sig = {
        "pl_graph_batch_create": (ctypes.c_int, [ctypes.c_int32, i32p, i32p, i32p, i32p,
                                                 ctypes.POINTER(vp)]),
        "pl_graph_batch_create_replicated": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, i32p, i32p,
                                                            ctypes.c_int32, ctypes.POINTER(vp)]),
        "pl_graph_batch_destroy": (ctypes.c_int, [vp]),
        "pl_graph_batch_info": (ctypes.c_int, [vp, i32p, i64p, i64p, i32p]),
        "pl_graph_batch_levels": (ctypes.c_int, [vp, i32p, i32p]),
        "pl_graph_batch_layout": (ctypes.c_int, [vp, i64p, i32p, i64p, i32p, i32p, i32p]),
        "pl_node_classes": (ctypes.c_int, [vp, vp, vp, vp]),
        "pl_debug_node_classes": (ctypes.c_int, [vp, vp, vp, vp]),
        "pl_weights_count": (ctypes.c_size_t, [cfgp]),
        "pl_weights_create": (ctypes.c_int, [cfgp, ctypes.POINTER(ctypes.c_float),
                                             ctypes.c_size_t, ctypes.POINTER(vp)]),
        "pl_weights_destroy": (ctypes.c_int, [vp]),
        "pl_weights_set_path": (ctypes.c_int, [vp, ctypes.c_int32]),
        "pl_embed_forward": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp]),
        "pl_embed_forward_ex": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]),
        "pl_graph_batch_upload": (ctypes.c_int, [vp]),
        "pl_embed_forward_static_limit": (ctypes.c_size_t, []),
        "pl_embed_forward_static_bytes": (ctypes.c_size_t, [vp, vp]),
        "pl_embed_forward_static": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, vp]),
        "pl_episode_step": (ctypes.c_int, [vp, ctypes.c_int32, vp, vp, vp, ctypes.c_int32, vp, vp, vp,
                                           vp, vp, vp]),
        "pl_episode_run": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                          vp, ctypes.c_int32, vp, vp, vp]),
        "pl_policy_gradient": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp, vp]),
        "pl_policy_gradient_ex": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, vp, vp, vp, vp, vp]),
        "pl_reinforce_coeff": (ctypes.c_int, [ctypes.c_int32, ctypes.c_int32, vp, vp, ctypes.c_int32, vp, vp, vp]),
        "pl_episode_gradient": (ctypes.c_int, [vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int32, ctypes.c_int32,
                                               ctypes.c_int32, vp, vp, vp, vp]),
        "pl_simulate_runtime": (ctypes.c_int, [vp, ctypes.c_int32, vp, vp, ctypes.c_float, vp, vp, vp]),
        "pl_simulate_runtime_ex": (ctypes.c_int, [vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_int32, vp, vp, vp]),
        "pl_simulate_reward_ex": (ctypes.c_int, [vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_int32,
                                                 ctypes.c_float, ctypes.c_float, vp, vp, vp, vp, vp]),
        "pl_simulate_reward": (ctypes.c_int, [vp, ctypes.c_int32, vp, vp, ctypes.c_float, ctypes.c_float,
                                              ctypes.c_float, vp, vp, vp, vp, vp]),
        "pl_profile_enable": (ctypes.c_int, [vp, ctypes.c_int32]),
        "pl_profile_read": (ctypes.c_int, [vp, ctypes.POINTER(ctypes.c_double), i64p,
                                           ctypes.c_int32]),
        "pl_last_error": (ctypes.c_char_p, []),
        "pl_version": (ctypes.c_char_p, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    if path == _LIB_PATH:
        _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        msg = load_library().pl_last_error().decode(errors="replace")
        raise PlacetoError(f"{what} failed ({rc}): {msg}")


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _dev_ptr(t, dtype, n_min, name):
    """Pointer of a contiguous torch tensor living on a HIP device."""
    import torch
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise PlacetoError(f"{name} must be a device tensor")
    if t.dtype != dtype or not t.is_contiguous() or t.numel() < n_min:
        raise PlacetoError(f"{name}: expected contiguous {dtype} with >= {n_min} elements, "
                           f"got {t.dtype} {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def weights_count(D, H, n_layers=2, k_sweeps=1, group_by_device=1, weight_dtype="fp32") -> int:
    cfg = ModelCfg(D, H, n_layers, k_sweeps, group_by_device, PL_WEIGHTS[weight_dtype], 0)
    return int(load_library().pl_weights_count(ctypes.byref(cfg)))


class GraphBatch:
    """pl_graph_batch: a batch of DAGs with its CSR, levels, buckets and scratch buffers."""

    def __init__(self, n_nodes, n_edges, edge_src, edge_dst, replicate=None):
        """replicate = R: n_nodes / n_edges are the sizes of ONE graph, and the batch holds R copies of
        it that share one layout (pl_graph_batch_create_replicated)."""
        lib = load_library()
        self._h = ctypes.c_void_p()
        src, ps = _i32(edge_src)
        dst, pd = _i32(edge_dst)
        if replicate is not None:
            if len(src) != len(dst) or len(src) != int(n_edges):
                raise PlacetoError("inconsistent graph arrays")
            _check(lib.pl_graph_batch_create_replicated(int(n_nodes), int(n_edges), ps, pd, int(replicate),
                                                        ctypes.byref(self._h)), "pl_graph_batch_create_replicated")
        else:
            n_nodes, pn = _i32(n_nodes)
            n_edges, pe = _i32(n_edges)
            if len(n_nodes) != len(n_edges) or len(src) != len(dst) or len(src) != int(n_edges.sum()):
                raise PlacetoError("inconsistent graph batch arrays")
            _check(lib.pl_graph_batch_create(len(n_nodes), pn, pe, ps, pd, ctypes.byref(self._h)),
                   "pl_graph_batch_create")
        B, n_tot, e_tot, depth = ctypes.c_int32(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        _check(lib.pl_graph_batch_info(self._h, ctypes.byref(B), ctypes.byref(n_tot),
                                       ctypes.byref(e_tot), ctypes.byref(depth)),
               "pl_graph_batch_info")
        self.B, self.n_tot, self.e_tot, self.max_depth = B.value, n_tot.value, e_tot.value, depth.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            load_library().pl_graph_batch_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def levels(self):
        td = np.zeros(self.n_tot, dtype=np.int32)
        bu = np.zeros(self.n_tot, dtype=np.int32)
        i32p = ctypes.POINTER(ctypes.c_int32)
        _check(load_library().pl_graph_batch_levels(self._h, td.ctypes.data_as(i32p),
                                                    bu.ctypes.data_as(i32p)),
               "pl_graph_batch_levels")
        return td, bu

    def layout(self):
        """dict of the host-side CSR and bucket orders (graph-local ids)."""
        i32p, i64p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64)
        out = dict(par_ptr=np.zeros(self.n_tot + 1, np.int64), par_idx=np.zeros(self.e_tot, np.int32),
                   chi_ptr=np.zeros(self.n_tot + 1, np.int64), chi_idx=np.zeros(self.e_tot, np.int32),
                   td_order=np.zeros(self.n_tot, np.int32), bu_order=np.zeros(self.n_tot, np.int32))
        _check(load_library().pl_graph_batch_layout(
            self._h, out["par_ptr"].ctypes.data_as(i64p), out["par_idx"].ctypes.data_as(i32p),
            out["chi_ptr"].ctypes.data_as(i64p), out["chi_idx"].ctypes.data_as(i32p),
            out["td_order"].ctypes.data_as(i32p), out["bu_order"].ctypes.data_as(i32p)),
            "pl_graph_batch_layout")
        return out

    def profile_enable(self, on: bool):
        _check(load_library().pl_profile_enable(self._h, 1 if on else 0), "pl_profile_enable")

    def profile_read(self, reset: bool = True):
        ms = (ctypes.c_double * len(STAGES))()
        cnt = (ctypes.c_int64 * len(STAGES))()
        _check(load_library().pl_profile_read(self._h, ms, cnt, 1 if reset else 0), "pl_profile_read")
        return {name: (ms[i], cnt[i]) for i, name in enumerate(STAGES)}


class Weights:
    """pl_weights: device copy of the parameter blob."""

    def __init__(self, blob, D, H, n_layers=2, k_sweeps=1, group_by_device=1, weight_dtype="fp32",
                 single_set=0):
        lib = load_library()
        self.cfg = ModelCfg(D, H, n_layers, k_sweeps, group_by_device, PL_WEIGHTS[weight_dtype], int(single_set))
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self._h = ctypes.c_void_p()
        _check(lib.pl_weights_create(ctypes.byref(self.cfg),
                                     blob.ctypes.data_as(ctypes.POINTER(ctypes.c_float)),
                                     blob.size, ctypes.byref(self._h)), "pl_weights_create")
        self.D, self.H, self.G = D, H, (D if group_by_device else 1)

    def set_path(self, path: int):
        """0 = fastest kernels available for this configuration, 1 = generic fp32 kernels."""
        _check(load_library().pl_weights_set_path(self._h, int(path)), "pl_weights_set_path")

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            load_library().pl_weights_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def node_classes(g: GraphBatch, cur_node, out_class, stream=None):
    """pl_node_classes: cur_node int32 [B] and out_class uint8 [N_tot], device tensors."""
    import torch
    _check(load_library().pl_node_classes(
        g._h, _dev_ptr(cur_node, torch.int32, g.B, "cur_node"),
        _dev_ptr(out_class, torch.uint8, g.n_tot, "out_class"), _stream_ptr(stream)),
        "pl_node_classes")
    return out_class


def embed_forward(g: GraphBatch, node_feats, placement, cur_node, w: Weights, out_logits,
                  out_probs=None, out_node_emb=None, out_pooled=None, stream=None, out_class=None):
    """pl_embed_forward / pl_embed_forward_ex on device tensors; asynchronous on `stream`
    (default: torch's current stream)."""
    import torch
    lib = load_library()
    args = [g._h,
            _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
            _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
            _dev_ptr(cur_node, torch.int32, g.B, "cur_node"),
            w._h,
            _dev_ptr(out_logits, torch.float32, g.B * w.D, "out_logits")]
    if out_probs is None and out_node_emb is None and out_pooled is None and out_class is None:
        _check(lib.pl_embed_forward(*args, _stream_ptr(stream)), "pl_embed_forward")
    else:
        _check(lib.pl_embed_forward_ex(
            *args, _dev_ptr(out_probs, torch.float32, g.B * w.D, "out_probs"),
            _dev_ptr(out_node_emb, torch.float32, g.n_tot * 2 * w.H, "out_node_emb"),
            _dev_ptr(out_pooled, torch.float32, g.B * 3 * w.G * w.H, "out_pooled"),
            _dev_ptr(out_class, torch.uint8, g.n_tot, "out_class"),
            _stream_ptr(stream)), "pl_embed_forward_ex")
    return out_logits


def graph_batch_upload(g: GraphBatch):
    """pl_graph_batch_upload: device copies of the batch's index data, made now."""
    _check(load_library().pl_graph_batch_upload(g._h), "pl_graph_batch_upload")


def embed_forward_static_limit() -> int:
    return int(load_library().pl_embed_forward_static_limit())


def embed_forward_static_bytes(g: GraphBatch, w: Weights) -> int:
    return int(load_library().pl_embed_forward_static_bytes(g._h, w._h))


def embed_forward_static(g: GraphBatch, node_feats, placement, cur_node, w: Weights, out_logits,
                         out_probs=None, stream=None):
    """pl_embed_forward_static on device tensors: the forward pass without any allocation."""
    import torch
    _check(load_library().pl_embed_forward_static(
        g._h, _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
        _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
        _dev_ptr(cur_node, torch.int32, g.B, "cur_node"), w._h,
        _dev_ptr(out_logits, torch.float32, g.B * w.D, "out_logits"),
        _dev_ptr(out_probs, torch.float32, g.B * w.D, "out_probs"), _stream_ptr(stream)),
        "pl_embed_forward_static")
    return out_logits


def episode_step(g: GraphBatch, D: int, logits, uniforms, order, t: int, node_feats, placement,
                 cur_node, out_action=None, out_logp=None, stream=None):
    """pl_episode_step on device tensors: one MDP transition for every graph, in place."""
    import torch
    lib = load_library()
    _check(lib.pl_episode_step(
        g._h, int(D), _dev_ptr(logits, torch.float32, g.B * D, "logits"),
        _dev_ptr(uniforms, torch.float32, g.B, "uniforms"),
        _dev_ptr(order, torch.int32, g.n_tot, "order"), int(t),
        _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
        _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
        _dev_ptr(cur_node, torch.int32, g.B, "cur_node"),
        _dev_ptr(out_action, torch.int32, g.B, "out_action"),
        _dev_ptr(out_logp, torch.float32, g.B, "out_logp"), _stream_ptr(stream)), "pl_episode_step")


def episode_run(g: GraphBatch, w: Weights, node_feats, placement, cur_node, order, uniforms,
                t0: int, n_steps: int, logits, keep_logits: bool = False, out_actions=None,
                out_logp=None, stream=None):
    """pl_episode_run on device tensors: n_steps x (forward pass, transition), in place and
    without host synchronisation."""
    import torch
    lib = load_library()
    n_log = g.B * w.D * (n_steps if keep_logits else 1)
    _check(lib.pl_episode_run(
        g._h, w._h, _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
        _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
        _dev_ptr(cur_node, torch.int32, g.B, "cur_node"),
        _dev_ptr(order, torch.int32, g.n_tot, "order"),
        _dev_ptr(uniforms, torch.float32, g.B * n_steps, "uniforms"), int(t0), int(n_steps),
        _dev_ptr(logits, torch.float32, n_log, "logits"), 1 if keep_logits else 0,
        _dev_ptr(out_actions, torch.int32, g.B * n_steps, "out_actions"),
        _dev_ptr(out_logp, torch.float32, g.B * n_steps, "out_logp"), _stream_ptr(stream)),
        "pl_episode_run")


def simulate_runtime(g: GraphBatch, D: int, node_feats, placement, inv_bandwidth: float, out_runtime,
                     out_events=None, stream=None, per_child_transfers=None):
    """pl_simulate_runtime(_ex) on device tensors: simulated run time of the placement of every graph."""
    import torch
    lib = load_library()
    head = [g._h, int(D), _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
            _dev_ptr(placement, torch.int32, g.n_tot, "placement"), float(inv_bandwidth)]
    tail = [_dev_ptr(out_runtime, torch.float32, g.B, "out_runtime"),
            _dev_ptr(out_events, torch.int32, g.B, "out_events"), _stream_ptr(stream)]
    if per_child_transfers is None:
        _check(lib.pl_simulate_runtime(*head, *tail), "pl_simulate_runtime")
    else:
        _check(lib.pl_simulate_runtime_ex(*head, int(per_child_transfers), *tail), "pl_simulate_runtime_ex")
    return out_runtime


def policy_gradient(g: GraphBatch, node_feats, placement, cur_node, w: Weights, actions, coeff, grad,
                    out_logits, out_logp=None, accumulate: bool = False, stream=None, entropy_coeff=None,
                    out_entropy=None):
    """pl_policy_gradient / pl_policy_gradient_ex on device tensors:
    grad (+)= sum_b coeff[b] * d log pi(a_b | s_b) / d theta (+ entropy_coeff[b] * d H(pi) / d theta)."""
    import torch
    lib = load_library()
    n_par = int(lib.pl_weights_count(ctypes.byref(w.cfg)))
    head = [g._h, _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
            _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
            _dev_ptr(cur_node, torch.int32, g.B, "cur_node"), w._h,
            _dev_ptr(actions, torch.int32, g.B, "actions"), _dev_ptr(coeff, torch.float32, g.B, "coeff")]
    tail = [1 if accumulate else 0, _dev_ptr(grad, torch.float32, n_par, "grad"),
            _dev_ptr(out_logits, torch.float32, g.B * w.D, "out_logits"),
            _dev_ptr(out_logp, torch.float32, g.B, "out_logp")]
    if entropy_coeff is None and out_entropy is None:
        _check(lib.pl_policy_gradient(*head, *tail, _stream_ptr(stream)), "pl_policy_gradient")
    else:
        _check(lib.pl_policy_gradient_ex(
            *head, _dev_ptr(entropy_coeff, torch.float32, g.B, "entropy_coeff"), *tail,
            _dev_ptr(out_entropy, torch.float32, g.B, "out_entropy"), _stream_ptr(stream)), "pl_policy_gradient_ex")
    return grad


def reinforce_coeff(rewards, group, n_groups: int, out_coeff, out_baseline=None, stream=None):
    """pl_reinforce_coeff on device tensors: rewards [T, B] -> return-minus-baseline weights [T, B]."""
    import torch
    lib = load_library()
    T, B = int(rewards.shape[0]), int(rewards.shape[1])
    _check(lib.pl_reinforce_coeff(
        T, B, _dev_ptr(rewards, torch.float32, T * B, "rewards"),
        _dev_ptr(group, torch.int32, B, "group"), int(n_groups),
        _dev_ptr(out_coeff, torch.float32, T * B, "out_coeff"),
        _dev_ptr(out_baseline, torch.float32, T * n_groups, "out_baseline"), _stream_ptr(stream)),
        "pl_reinforce_coeff")
    return out_coeff


def episode_gradient(g: GraphBatch, w: Weights, node_feats, placement, cur_node, order, actions, coeff,
                     t0: int, n_steps: int, grad, logits, out_logp=None, accumulate: bool = False, stream=None,
                     entropy_coeff=None):
    """pl_episode_gradient on device tensors: the REINFORCE sum over n_steps recorded steps."""
    import torch
    lib = load_library()
    n_par = int(lib.pl_weights_count(ctypes.byref(w.cfg)))
    _check(lib.pl_episode_gradient(
        g._h, w._h, _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
        _dev_ptr(placement, torch.int32, g.n_tot, "placement"),
        _dev_ptr(cur_node, torch.int32, g.B, "cur_node"),
        _dev_ptr(order, torch.int32, g.n_tot, "order"),
        _dev_ptr(actions, torch.int32, g.B * n_steps, "actions"),
        _dev_ptr(coeff, torch.float32, g.B * n_steps, "coeff"),
        _dev_ptr(entropy_coeff, torch.float32, g.B * n_steps, "entropy_coeff"), int(t0), int(n_steps),
        1 if accumulate else 0, _dev_ptr(grad, torch.float32, n_par, "grad"),
        _dev_ptr(logits, torch.float32, g.B * w.D, "logits"),
        _dev_ptr(out_logp, torch.float32, g.B * n_steps, "out_logp"), _stream_ptr(stream)),
        "pl_episode_gradient")
    return grad


def simulate_reward(g: GraphBatch, D: int, node_feats, placement, inv_bandwidth: float, mem_limit: float,
                    mem_penalty: float, out_reward, out_runtime=None, out_peak_mem=None, out_events=None,
                    stream=None, per_child_transfers=None):
    """pl_simulate_reward(_ex) on device tensors: memory-penalised run time R(p) of every graph's placement."""
    import torch
    lib = load_library()
    head = [g._h, int(D), _dev_ptr(node_feats, torch.float32, g.n_tot * 3, "node_feats"),
            _dev_ptr(placement, torch.int32, g.n_tot, "placement"), float(inv_bandwidth)]
    tail = [float(mem_limit), float(mem_penalty), _dev_ptr(out_reward, torch.float32, g.B, "out_reward"),
            _dev_ptr(out_runtime, torch.float32, g.B, "out_runtime"),
            _dev_ptr(out_peak_mem, torch.float32, g.B * D, "out_peak_mem"),
            _dev_ptr(out_events, torch.int32, g.B, "out_events"), _stream_ptr(stream)]
    if per_child_transfers is None:
        _check(lib.pl_simulate_reward(*head, *tail), "pl_simulate_reward")
    else:
        _check(lib.pl_simulate_reward_ex(*head, int(per_child_transfers), *tail), "pl_simulate_reward_ex")
    return out_reward
