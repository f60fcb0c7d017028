"""ctypes binding of librefreshkv.so: same names as the C ABI, torch tensors for device memory.

Argument marshalling only.  Shapes and dtypes are checked here so that a wrong tensor is an
exception on the host and never a bad pointer on the GPU.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "librefreshkv.so")

EXPORTS = ["rk_version", "rk_status_string", "rk_workspace_bytes", "rk_workspace_init",
           "rk_full_attn", "rk_full_attn_scores", "rk_topk_select", "rk_full_attn_select", "rk_full_attn_pool", "rk_full_attn_deferred", "rk_select_pooled", "rk_score_select", "rk_window_select", "rk_gather_small_kv", "rk_partial_attn", "rk_partial_attn_static", "rk_partial_attn_static_bytes", "rk_partial_attn_fixed", "rk_partial_attn_lazy", "rk_partial_attn_triggered", "rk_decode_step", "rk_decode_step_overlapped", "rk_refresh_batched", "rk_decode_step_batched",
           "rk_query_sim", "rk_mark_refresh", "rk_calibration_copy", "rk_calibration_read", "rk_debug_set_slice_spin", "rk_h2o_append", "rk_h2o_update", "rk_h2o_step"]

RK_AGG_MAX, RK_AGG_MEAN, RK_AGG_FIRST = 0, 1, 2


class RkError(RuntimeError):
    def __init__(self, fn: str, status: int):
        super().__init__("%s failed: %s (%d)" % (fn, status_string(status), status))
        self.status = status


class _Geom(C.Structure):
    _fields_ = [("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("scale", C.c_float)]


class _Kv(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("stride_b", C.c_int64), ("stride_h", C.c_int64),
                ("capacity", C.c_int64)]


class _LayerState(C.Structure):
    _fields_ = [("full", _Kv), ("small", _Kv), ("idx", C.c_void_p), ("tail_start", C.c_void_p),
                ("q_ref", C.c_void_p), ("sim", C.c_void_p), ("need_full", C.c_void_p), ("n_full", C.c_void_p)]


class _H2oState(C.Structure):
    _fields_ = [("cache", _Kv), ("total", C.c_void_p), ("pos", C.c_void_p), ("n_rows", C.c_void_p),
                ("n_attend", C.c_void_p)]


class _Schedule(C.Structure):
    _fields_ = [("k", C.c_int32), ("pool_w", C.c_int32), ("stride", C.c_int32), ("dynamic", C.c_int32),
                ("threshold", C.c_float), ("fixed_size", C.c_int32), ("scores_only", C.c_int32)]


class _Overlap(C.Structure):
    _fields_ = [("side_stream", C.c_void_p), ("ready", C.POINTER(C.c_void_p)), ("done", C.POINTER(C.c_void_p)),
                ("join", C.c_void_p), ("workspaces", C.POINTER(C.c_void_p)), ("n_workspaces", C.c_int32),
                ("workspace_bytes", C.c_size_t)]


STEP_KINDS = {1: "full", 2: "partial", 3: "both"}


def _load(path: str = LIB_PATH) -> C.CDLL:
    if not os.path.exists(path):
        raise ImportError("librefreshkv.so is not built (%s missing); run "
                          "`python paper_2411_05787_amd/build.py` first. There is no fallback path." % path)
    l = C.CDLL(path)
    P, I32, I64, SZ = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    G = C.POINTER(_Geom)
    l.rk_version.restype = C.c_int
    l.rk_version.argtypes = []
    l.rk_status_string.restype = C.c_char_p
    l.rk_status_string.argtypes = [C.c_int]
    l.rk_workspace_bytes.restype = SZ
    l.rk_workspace_bytes.argtypes = [G, I32, I32]
    l.rk_workspace_init.restype = C.c_int
    l.rk_workspace_init.argtypes = [G, P, SZ, P]
    l.rk_full_attn.restype = C.c_int
    l.rk_full_attn.argtypes = [G, P, _Kv, P, I32, P, P, I64, P, P, I32, P, SZ, P]
    l.rk_full_attn_scores.restype = C.c_int
    l.rk_full_attn_scores.argtypes = [G, P, _Kv, P, I32, P, I64, P, I32, P, SZ, P]
    l.rk_topk_select.restype = C.c_int
    l.rk_topk_select.argtypes = [G, P, I64, P, I32, I32, I32, I32, P, P, P, I32, P, SZ, P]
    l.rk_gather_small_kv.restype = C.c_int
    l.rk_full_attn_select.argtypes = [G, P, _Kv, P, I32, P, P, I64, P, I32, I32, I32, P, P, P, I32, P, SZ, P]
    l.rk_full_attn_select.restype = C.c_int
    l.rk_full_attn_pool.restype = C.c_int
    l.rk_full_attn_deferred.restype = C.c_int
    l.rk_full_attn_deferred.argtypes = [G, P, _Kv, P, I32, P, P, P, I32, P, SZ, P]
    l.rk_full_attn_pool.argtypes = [G, P, _Kv, P, I32, P, P, I64, P, I32, I32, I32, P, I32, P, SZ, P]
    l.rk_select_pooled.restype = C.c_int
    l.rk_select_pooled.argtypes = [G, P, I32, I32, P, P, P, I32, P, SZ, P]
    l.rk_score_select.argtypes = [G, P, _Kv, P, I32, P, I64, P, I32, I32, I32, P, P, P, I32, P, SZ, P]
    l.rk_score_select.restype = C.c_int
    l.rk_window_select.argtypes = [G, P, I32, _Kv, P, I32, P, I64, I32, I32, I32, P, P, P, I32, P, SZ, P]
    l.rk_window_select.restype = C.c_int
    l.rk_gather_small_kv.argtypes = [G, _Kv, P, I32, _Kv, P, P, P, I32, P]
    l.rk_partial_attn.restype = C.c_int
    l.rk_partial_attn.argtypes = [G, P, _Kv, I32, _Kv, P, P, I32, P, P, I32, P, SZ, P]
    l.rk_partial_attn_static.restype = C.c_int
    l.rk_partial_attn_static.argtypes = [G, P, _Kv, I32, _Kv, P, P, I32, P, P, I32, P]
    l.rk_partial_attn_static_bytes.restype = SZ
    l.rk_partial_attn_static_bytes.argtypes = [G, I32, I32]
    l.rk_partial_attn_fixed.restype = C.c_int
    l.rk_partial_attn_fixed.argtypes = [G, P, _Kv, I32, _Kv, P, P, I32, P, P, I32, P, SZ, P]
    l.rk_partial_attn_lazy.argtypes = [G, P, _Kv, P, I32, I32, _Kv, P, P, I32, P, P, I32, P, SZ, P]
    l.rk_partial_attn_lazy.restype = C.c_int
    l.rk_query_sim.restype = C.c_int
    l.rk_partial_attn_triggered.restype = C.c_int
    l.rk_partial_attn_triggered.argtypes = [G, P, _Kv, I32, I32, _Kv, P, P, I32, P, P, C.c_float, P, P, P, SZ, P]
    l.rk_decode_step.restype = C.c_int
    l.rk_decode_step.argtypes = [G, C.POINTER(_Schedule), I32, I32, C.POINTER(_LayerState), C.POINTER(C.c_void_p),
                                 C.POINTER(C.c_void_p), P, I32, I32, P, SZ, P]
    l.rk_decode_step_overlapped.restype = C.c_int
    l.rk_decode_step_overlapped.argtypes = [G, C.POINTER(_Schedule), I32, I32, C.POINTER(_LayerState), C.POINTER(C.c_void_p),
                                            C.POINTER(C.c_void_p), P, I32, I32, C.POINTER(_Overlap), P]
    l.rk_decode_step_batched.argtypes = [G, C.POINTER(_Schedule), I32, I32, C.POINTER(_LayerState), C.POINTER(C.c_void_p),
                                         C.POINTER(C.c_void_p), P, I32, I32, C.POINTER(C.c_void_p), SZ, P]
    l.rk_decode_step_batched.restype = C.c_int
    l.rk_refresh_batched.argtypes = [G, I32, C.POINTER(_LayerState), C.POINTER(C.c_void_p), SZ, P, I32, I32, I32, I32, I32, P]
    l.rk_refresh_batched.restype = C.c_int
    l.rk_query_sim.argtypes = [G, P, P, C.c_float, I32, P, P, P]
    l.rk_calibration_copy.restype = C.c_int
    l.rk_calibration_copy.argtypes = [P, P, SZ, P]
    l.rk_debug_set_slice_spin.restype = C.c_int
    l.rk_debug_set_slice_spin.argtypes = [C.c_int32]
    l.rk_calibration_read.restype = C.c_int
    l.rk_calibration_read.argtypes = [P, SZ, P, P]
    l.rk_mark_refresh.restype = C.c_int
    l.rk_mark_refresh.argtypes = [G, P, P, P, I32, P]
    l.rk_h2o_append.argtypes = [G, _H2oState, P, P, P, I32, P]
    l.rk_h2o_append.restype = C.c_int
    l.rk_h2o_update.argtypes = [G, _H2oState, P, I64, I32, I32, I32, P, P]
    l.rk_h2o_update.restype = C.c_int
    l.rk_h2o_step.argtypes = [G, _H2oState, P, P, P, P, I32, I32, I32, P, P, P, SZ, P]
    l.rk_h2o_step.restype = C.c_int
    return l


lib = _load()


def version() -> int:
    return int(lib.rk_version())


def status_string(status: int) -> str:
    return lib.rk_status_string(int(status)).decode()


@dataclass(frozen=True)
class Geom:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    scale: float

    def c(self) -> _Geom:
        return _Geom(self.batch, self.n_q_heads, self.n_kv_heads, self.head_dim, self.scale)


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise RkError(fn, rc)


def _dev(t: Optional[torch.Tensor], dtype, name: str, shape=None, optional=False) -> Optional[int]:
    if t is None:
        if optional:
            return None
        raise ValueError("%s is required" % name)
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError("%s must be a tensor in GPU memory" % name)
    if t.dtype != dtype:
        raise ValueError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


def _kv(geom: Geom, K: torch.Tensor, V: torch.Tensor, name: str, min_rows: int = 0) -> _Kv:
    for t, n in ((K, name + ".k"), (V, name + ".v")):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or t.dtype != torch.bfloat16:
            raise ValueError("%s must be a bf16 tensor in GPU memory" % n)
        if t.dim() != 4 or t.shape[0] != geom.batch or t.shape[1] != geom.n_kv_heads or t.shape[3] != geom.head_dim:
            raise ValueError("%s must be [batch, n_kv_heads, capacity, head_dim], got %s" % (n, tuple(t.shape)))
        if t.stride(3) != 1 or t.stride(2) != geom.head_dim:
            raise ValueError("%s rows must be contiguous" % n)
        if t.shape[2] < min_rows:
            raise ValueError("%s holds %d rows, %d needed" % (n, t.shape[2], min_rows))
    if K.stride() != V.stride() or K.shape != V.shape:
        raise ValueError("%s: k and v must share shape and strides" % name)
    return _Kv(K.data_ptr(), V.data_ptr(), K.stride(0), K.stride(1), K.shape[2])


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def workspace_bytes(geom: Geom, max_len: int, max_k: int) -> int:
    n = int(lib.rk_workspace_bytes(C.byref(geom.c()), int(max_len), int(max_k)))
    if n == 0:
        raise RkError("rk_workspace_bytes", -1)
    return n


class Workspace:
    """Device scratch for one stream: allocated once, initialised once."""

    def __init__(self, geom: Geom, max_len: int, max_k: int, device="cuda", stream=None):
        self.geom = geom
        self.max_len = int(max_len)
        self.nbytes = workspace_bytes(geom, max_len, max_k)
        self.buf = torch.empty(self.nbytes + 256, dtype=torch.uint8, device=device)
        self.ptr = (self.buf.data_ptr() + 255) // 256 * 256
        rk_workspace_init(geom, self, stream=stream)


def rk_workspace_init(geom: Geom, ws: Workspace, stream=None) -> None:
    _check("rk_workspace_init", lib.rk_workspace_init(C.byref(geom.c()), ws.ptr, ws.nbytes, _stream(stream)))


def rk_full_attn(geom: Geom, q, K, V, seq_lens, max_len: int, out, weights=None, lse=None,
                 pred=None, pred_val: int = 0, workspace: Workspace = None, stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    w_stride = 0
    if weights is not None:
        if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq or weights.shape[2] < max_len:
            raise ValueError("weights must be [batch, n_q_heads, >= max_len]")
        w_stride = weights.shape[2]
    _check("rk_full_attn", lib.rk_full_attn(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _kv(geom, K, V, "full"),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(weights, torch.float32, "weights", optional=True), w_stride,
        _dev(lse, torch.float32, "lse", (B, Hq), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_full_attn_scores(geom: Geom, q, K, V, seq_lens, max_len: int, scores=None, pred=None, pred_val: int = 0,
                        workspace: Workspace = None, stream=None) -> None:
    """scores=None: the raw scores stay in the workspace (the first kernel of a full step, as the
    refreshing calls launch it)."""
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    if scores is not None and (scores.dim() != 3 or scores.shape[0] != B or scores.shape[1] != Hq or scores.shape[2] < max_len):
        raise ValueError("scores must be [batch, n_q_heads, >= max_len]")
    _check("rk_full_attn_scores", lib.rk_full_attn_scores(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _kv(geom, K, V, "full"),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(scores, torch.float32, "scores", optional=True), scores.shape[2] if scores is not None else 0,
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_topk_select(geom: Geom, weights, seq_lens, max_len: int, k: int, pool_w: int, idx,
                   sel_scores=None, agg: int = RK_AGG_MAX, pred=None, pred_val: int = 0,
                   workspace: Workspace = None, stream=None) -> None:
    B, Hq, Hkv = geom.batch, geom.n_q_heads, geom.n_kv_heads
    if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq or weights.shape[2] < max_len:
        raise ValueError("weights must be [batch, n_q_heads, >= max_len]")
    _check("rk_topk_select", lib.rk_topk_select(
        C.byref(geom.c()), _dev(weights, torch.float32, "weights"), weights.shape[2],
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len), int(k), int(pool_w), int(agg),
        _dev(idx, torch.int32, "idx", (B, Hkv, k)),
        _dev(sel_scores, torch.float32, "sel_scores", (B, Hkv, k), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_full_attn_select(geom: Geom, q, K, V, seq_lens, max_len: int, out, k: int, pool_w: int, idx,
                        weights=None, lse=None, sel_scores=None, agg: int = RK_AGG_MAX,
                        pred=None, pred_val: int = 0, workspace: Workspace = None, stream=None) -> None:
    B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    w_stride = 0
    if weights is not None:
        if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq or weights.shape[2] < max_len:
            raise ValueError("weights must be [batch, n_q_heads, >= max_len]")
        w_stride = weights.shape[2]
    _check("rk_full_attn_select", lib.rk_full_attn_select(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _kv(geom, K, V, "full"),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(weights, torch.float32, "weights", optional=True), w_stride,
        _dev(lse, torch.float32, "lse", (B, Hq), optional=True),
        int(k), int(pool_w), int(agg),
        _dev(idx, torch.int32, "idx", (B, Hkv, k)),
        _dev(sel_scores, torch.float32, "sel_scores", (B, Hkv, k), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_full_attn_pool(geom: Geom, q, K, V, seq_lens, max_len: int, out, pool_w: int, weights=None, lse=None,
                      agg: int = RK_AGG_MAX, pred=None, pred_val: int = 0, workspace: Workspace = None,
                      stream=None, beside_other_work: bool = False) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    w_stride = 0
    if weights is not None:
        if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq or weights.shape[2] < max_len:
            raise ValueError("weights must be [batch, n_q_heads, >= max_len]")
        w_stride = weights.shape[2]
    _check("rk_full_attn_pool", lib.rk_full_attn_pool(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _kv(geom, K, V, "full"),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(weights, torch.float32, "weights", optional=True), w_stride,
        _dev(lse, torch.float32, "lse", (B, Hq), optional=True), int(pool_w), int(agg), int(bool(beside_other_work)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_full_attn_deferred(geom: Geom, q, K, V, seq_lens, max_len: int, out, lse=None, pred=None, pred_val: int = 0,
                          workspace: Workspace = None, stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    _check("rk_full_attn_deferred", lib.rk_full_attn_deferred(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _kv(geom, K, V, "full"),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(lse, torch.float32, "lse", (B, Hq), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_select_pooled(geom: Geom, seq_lens, max_len: int, k: int, idx, sel_scores=None, pred=None, pred_val: int = 0,
                     workspace: Workspace = None, stream=None) -> None:
    B, Hkv = geom.batch, geom.n_kv_heads
    _check("rk_select_pooled", lib.rk_select_pooled(
        C.byref(geom.c()), _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len), int(k),
        _dev(idx, torch.int32, "idx", (B, Hkv, k)),
        _dev(sel_scores, torch.float32, "sel_scores", (B, Hkv, k), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_score_select(geom: Geom, q, K, seq_lens, max_len: int, k: int, pool_w: int, idx,
                    weights=None, lse=None, sel_scores=None, agg: int = RK_AGG_MAX,
                    pred=None, pred_val: int = 0, workspace: Workspace = None, stream=None) -> None:
    """K: bf16 [B, Hkv, capacity, D]; the values of the full cache are not needed."""
    B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    w_stride = 0
    if weights is not None:
        if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq or weights.shape[2] < max_len:
            raise ValueError("weights must be [batch, n_q_heads, >= max_len]")
        w_stride = weights.shape[2]
    kv = _kv(geom, K, K, "full")
    kv.v = None
    _check("rk_score_select", lib.rk_score_select(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), kv,
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(weights, torch.float32, "weights", optional=True), w_stride,
        _dev(lse, torch.float32, "lse", (B, Hq), optional=True),
        int(k), int(pool_w), int(agg),
        _dev(idx, torch.int32, "idx", (B, Hkv, k)),
        _dev(sel_scores, torch.float32, "sel_scores", (B, Hkv, k), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_window_select(geom: Geom, q_win, K, seq_lens, max_len: int, k: int, pool_w: int, idx,
                     votes=None, sel_scores=None, agg: int = RK_AGG_MAX,
                     pred=None, pred_val: int = 0, workspace: Workspace = None, stream=None) -> None:
    """q_win: bf16 [B, W, Hq, D], the queries of the last W prompt tokens; K: bf16 [B, Hkv, capacity, D]."""
    B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
    if q_win.dim() != 4:
        raise ValueError("q_win must be [batch, window, n_q_heads, head_dim]")
    W = q_win.shape[1]
    if max_len > K.shape[2]:
        raise ValueError("max_len %d exceeds the cache capacity %d" % (max_len, K.shape[2]))
    v_stride = 0
    if votes is not None:
        if votes.dim() != 3 or votes.shape[0] != B or votes.shape[1] != Hq or votes.shape[2] < max_len:
            raise ValueError("votes must be [batch, n_q_heads, >= max_len]")
        v_stride = votes.shape[2]
    kv = _kv(geom, K, K, "full")
    kv.v = None
    _check("rk_window_select", lib.rk_window_select(
        C.byref(geom.c()), _dev(q_win, torch.bfloat16, "q_win", (B, W, Hq, D)), int(W), kv,
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(max_len),
        _dev(votes, torch.float32, "votes", optional=True), v_stride,
        int(k), int(pool_w), int(agg),
        _dev(idx, torch.int32, "idx", (B, Hkv, k)),
        _dev(sel_scores, torch.float32, "sel_scores", (B, Hkv, k), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_gather_small_kv(geom: Geom, K, V, idx, k: int, small_K, small_V, seq_lens=None, tail_start=None,
                       pred=None, pred_val: int = 0, stream=None) -> None:
    B, Hkv = geom.batch, geom.n_kv_heads
    _check("rk_gather_small_kv", lib.rk_gather_small_kv(
        C.byref(geom.c()), _kv(geom, K, V, "full"), _dev(idx, torch.int32, "idx", (B, Hkv, k)), int(k),
        _kv(geom, small_K, small_V, "small", min_rows=k),
        _dev(seq_lens, torch.int32, "seq_lens", (B,), optional=True),
        _dev(tail_start, torch.int32, "tail_start", (B,), optional=True),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val), _stream(stream)))


def rk_partial_attn(geom: Geom, q, small_K, small_V, n_sel: int, K, V, tail_start, seq_lens,
                    max_recent: int, out, pred=None, pred_val: int = 0, workspace: Workspace = None,
                    stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    _check("rk_partial_attn", lib.rk_partial_attn(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _kv(geom, small_K, small_V, "small", min_rows=n_sel), int(n_sel), _kv(geom, K, V, "full"),
        _dev(tail_start, torch.int32, "tail_start", (B,)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(max_recent), _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


STATIC_SCRATCH_BYTES = 8 << 20


def rk_partial_attn_static_bytes(geom: Geom, n_sel: int, max_recent: int) -> int:
    return int(lib.rk_partial_attn_static_bytes(C.byref(geom.c()), int(n_sel), int(max_recent)))


def rk_partial_attn_static(geom: Geom, q, small_K, small_V, n_sel: int, K, V, tail_start, seq_lens,
                           max_recent: int, out, pred=None, pred_val: int = 0, stream=None) -> None:
    """rk_partial_attn on the library's built-in scratch array: no workspace, nothing allocated."""
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    _check("rk_partial_attn_static", lib.rk_partial_attn_static(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _kv(geom, small_K, small_V, "small", min_rows=n_sel), int(n_sel), _kv(geom, K, V, "full"),
        _dev(tail_start, torch.int32, "tail_start", (B,)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(max_recent), _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val), _stream(stream)))


def rk_partial_attn_fixed(geom: Geom, q, small_K, small_V, k: int, K, V, tail_start, seq_lens,
                          max_recent: int, out, pred=None, pred_val: int = 0, workspace: Workspace = None,
                          stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    _check("rk_partial_attn_fixed", lib.rk_partial_attn_fixed(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _kv(geom, small_K, small_V, "small", min_rows=k), int(k), _kv(geom, K, V, "full"),
        _dev(tail_start, torch.int32, "tail_start", (B,)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(max_recent), _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_partial_attn_lazy(geom: Geom, q, small_K, small_V, idx, k: int, K, V, tail_start, seq_lens,
                         max_recent: int, out, fixed_size: bool = False, pred=None, pred_val: int = 0,
                         workspace: Workspace = None, stream=None) -> None:
    """The first partial step after a refresh without a gather: selected rows come from (K, V) through
    idx and are written into (small_K, small_V) on the way."""
    B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
    _check("rk_partial_attn_lazy", lib.rk_partial_attn_lazy(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _kv(geom, small_K, small_V, "small", min_rows=k), _dev(idx, torch.int32, "idx", (B, Hkv, k)), int(k),
        int(bool(fixed_size)), _kv(geom, K, V, "full"),
        _dev(tail_start, torch.int32, "tail_start", (B,)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(max_recent), _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def layer_state(geom: Geom, K, V, small_K, small_V, idx, tail_start, q_ref=None, sim=None, need_full=None,
                n_full=None, k: int = 0) -> _LayerState:
    """One entry of rk_decode_step's `layers` array (the tensors must outlive its use)."""
    B, Hkv, D = geom.batch, geom.n_kv_heads, geom.head_dim
    return _LayerState(_kv(geom, K, V, "full"), _kv(geom, small_K, small_V, "small", min_rows=k),
                       _dev(idx, torch.int32, "idx", (B, Hkv, k) if k else None),
                       _dev(tail_start, torch.int32, "tail_start", (B,)),
                       _dev(q_ref, torch.float32, "q_ref", (B, D), optional=True),
                       _dev(sim, torch.float32, "sim", (B,), optional=True),
                       _dev(need_full, torch.int32, "need_full", (B,), optional=True),
                       _dev(n_full, torch.int32, "n_full", (B,), optional=True))


def rk_decode_step(geom: Geom, sched: _Schedule, t: int, layers, q_ptrs, out_ptrs, seq_lens, max_len: int,
                   max_recent: int, workspace: Workspace = None, stream=None) -> str:
    """layers: ctypes array of _LayerState; q_ptrs / out_ptrs: ctypes arrays of device pointers
    (one per layer).  Returns "full", "partial" or "both"."""
    n = len(layers)
    rc = lib.rk_decode_step(C.byref(geom.c()), C.byref(sched), int(t), n, layers, q_ptrs, out_ptrs,
                            _dev(seq_lens, torch.int32, "seq_lens", (geom.batch,)), int(max_len), int(max_recent),
                            workspace.ptr, workspace.nbytes, _stream(stream))
    if rc <= 0:
        _check("rk_decode_step", rc if rc < 0 else -1)
    return STEP_KINDS[rc]


def rk_decode_step_overlapped(geom: Geom, sched: _Schedule, t: int, layers, q_ptrs, out_ptrs, seq_lens, max_len: int,
                              max_recent: int, overlap: _Overlap, stream=None) -> str:
    rc = lib.rk_decode_step_overlapped(C.byref(geom.c()), C.byref(sched), int(t), len(layers), layers, q_ptrs, out_ptrs,
                                       _dev(seq_lens, torch.int32, "seq_lens", (geom.batch,)), int(max_len),
                                       int(max_recent), C.byref(overlap), _stream(stream))
    if rc <= 0:
        _check("rk_decode_step_overlapped", rc if rc < 0 else -1)
    return STEP_KINDS[rc]


def rk_partial_attn_triggered(geom: Geom, q, small_K, small_V, n_sel: int, K, V, tail_start, seq_lens,
                              max_recent: int, out, q_ref, threshold: float, sim, need_full,
                              fixed_size: bool = False, workspace: Workspace = None, stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    _check("rk_partial_attn_triggered", lib.rk_partial_attn_triggered(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _kv(geom, small_K, small_V, "small", min_rows=n_sel), int(n_sel), 1 if fixed_size else 0, _kv(geom, K, V, "full"),
        _dev(tail_start, torch.int32, "tail_start", (B,)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(max_recent), _dev(out, torch.bfloat16, "out", (B, Hq, D)),
        _dev(q_ref, torch.float32, "q_ref", (B, D)), float(threshold), _dev(sim, torch.float32, "sim", (B,)),
        _dev(need_full, torch.int32, "need_full", (B,)), workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_query_sim(geom: Geom, q, q_ref, threshold: float, force_full: bool, sim, need_full, stream=None) -> None:
    B, Hq, D = geom.batch, geom.n_q_heads, geom.head_dim
    _check("rk_query_sim", lib.rk_query_sim(
        C.byref(geom.c()), _dev(q, torch.bfloat16, "q", (B, Hq, D)), _dev(q_ref, torch.float32, "q_ref", (B, D)),
        float(threshold), 1 if force_full else 0, _dev(sim, torch.float32, "sim", (B,)),
        _dev(need_full, torch.int32, "need_full", (B,)), _stream(stream)))


def rk_mark_refresh(geom: Geom, seq_lens, tail_start, pred=None, pred_val: int = 0, stream=None) -> None:
    B = geom.batch
    _check("rk_mark_refresh", lib.rk_mark_refresh(
        C.byref(geom.c()), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        _dev(tail_start, torch.int32, "tail_start", (B,)),
        _dev(pred, torch.int32, "pred", (B,), optional=True), int(pred_val), _stream(stream)))


def rk_debug_set_slice_spin(spin: int) -> None:
    """Test hook: how often a workgroup of the merge by slices re-reads rows still in flight before it hands its
    share over (default 256; 0: every workgroup hands over at once).  Results do not depend on it."""
    _check("rk_debug_set_slice_spin", lib.rk_debug_set_slice_spin(int(spin)))


def rk_calibration_read(src: torch.Tensor, sink: torch.Tensor, nbytes: int = None, offset: int = 0, stream=None) -> int:
    """Reads nbytes of src from byte `offset` on (default: all of it) and keeps nothing; returns the bytes read.
    sink: one int32 in GPU memory."""
    if not isinstance(src, torch.Tensor) or not src.is_cuda or not src.is_contiguous():
        raise ValueError("src must be a contiguous tensor in GPU memory")
    total = src.numel() * src.element_size()
    nbytes = total - offset if nbytes is None else int(nbytes)
    if offset < 0 or nbytes <= 0 or offset + nbytes > total or offset % 16 or nbytes % 16:
        raise ValueError("the range read must lie inside src and be a multiple of 16 bytes")
    _check("rk_calibration_read", lib.rk_calibration_read(src.data_ptr() + offset, nbytes,
                                                          _dev(sink, torch.int32, "sink", (1,)), _stream(stream)))
    return nbytes


def rk_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> int:
    """Copies src to dst (same byte size, contiguous GPU tensors); returns the bytes copied."""
    for t, n in ((dst, "dst"), (src, "src")):
        if not isinstance(t, torch.Tensor) or not t.is_cuda or not t.is_contiguous():
            raise ValueError("%s must be a contiguous tensor in GPU memory" % n)
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("dst and src must have the same size in bytes")
    _check("rk_calibration_copy", lib.rk_calibration_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream(stream)))
    return nbytes


def h2o_state(geom: Geom, cache_K, cache_V, total, pos, n_rows, n_attend) -> _H2oState:
    """The H2O policy's state as the C struct (the tensors must outlive its use).  cache_K/V bf16
    [B, Hkv, capacity, D]; total fp32 and pos int32 [B, Hkv, capacity]; n_rows, n_attend int32 [B]."""
    B, Hkv = geom.batch, geom.n_kv_heads
    cap = cache_K.shape[2]
    return _H2oState(_kv(geom, cache_K, cache_V, "cache"),
                     _dev(total, torch.float32, "total", (B, Hkv, cap)), _dev(pos, torch.int32, "pos", (B, Hkv, cap)),
                     _dev(n_rows, torch.int32, "n_rows", (B,)), _dev(n_attend, torch.int32, "n_attend", (B,)))


def rk_h2o_append(geom: Geom, state: _H2oState, k_new, v_new, seq_lens, budget: int, stream=None) -> None:
    B, Hkv, D = geom.batch, geom.n_kv_heads, geom.head_dim
    _check("rk_h2o_append", lib.rk_h2o_append(
        C.byref(geom.c()), state, _dev(k_new, torch.bfloat16, "k_new", (B, Hkv, D)),
        _dev(v_new, torch.bfloat16, "v_new", (B, Hkv, D)), _dev(seq_lens, torch.int32, "seq_lens", (B,)),
        int(budget), _stream(stream)))


def rk_h2o_update(geom: Geom, state: _H2oState, weights, budget: int, recent: int, agg: int = RK_AGG_MAX,
                  dropped=None, stream=None) -> None:
    B, Hq, Hkv = geom.batch, geom.n_q_heads, geom.n_kv_heads
    if weights.dim() != 3 or weights.shape[0] != B or weights.shape[1] != Hq:
        raise ValueError("weights must be [batch, n_q_heads, >= budget + 1]")
    _check("rk_h2o_update", lib.rk_h2o_update(
        C.byref(geom.c()), state, _dev(weights, torch.float32, "weights"), weights.shape[2],
        int(budget), int(recent), int(agg), _dev(dropped, torch.int32, "dropped", (B, Hkv), optional=True),
        _stream(stream)))


def rk_h2o_step(geom: Geom, state: _H2oState, q, k_new, v_new, seq_lens, budget: int, recent: int, out,
                agg: int = RK_AGG_MAX, dropped=None, workspace: Workspace = None, stream=None) -> None:
    B, Hq, Hkv, D = geom.batch, geom.n_q_heads, geom.n_kv_heads, geom.head_dim
    _check("rk_h2o_step", lib.rk_h2o_step(
        C.byref(geom.c()), state, _dev(q, torch.bfloat16, "q", (B, Hq, D)),
        _dev(k_new, torch.bfloat16, "k_new", (B, Hkv, D)), _dev(v_new, torch.bfloat16, "v_new", (B, Hkv, D)),
        _dev(seq_lens, torch.int32, "seq_lens", (B,)), int(budget), int(recent), int(agg),
        _dev(out, torch.bfloat16, "out", (B, Hq, D)), _dev(dropped, torch.int32, "dropped", (B, Hkv), optional=True),
        workspace.ptr, workspace.nbytes, _stream(stream)))


def rk_refresh_batched(geom: Geom, layers, ws_ptrs, workspace_bytes: int, seq_lens, max_len: int, k: int,
                       pool_w: int = 0, agg: int = RK_AGG_MAX, by_need_full: bool = False, stream=None) -> None:
    """layers: ctypes array of _LayerState; ws_ptrs: ctypes array of one workspace pointer per layer.
    pool_w != 0: the layers ran rk_full_attn_deferred and are pooled here first."""
    _check("rk_refresh_batched", lib.rk_refresh_batched(
        C.byref(geom.c()), len(layers), layers, ws_ptrs, int(workspace_bytes),
        _dev(seq_lens, torch.int32, "seq_lens", (geom.batch,)), int(max_len), int(k), int(pool_w), int(agg),
        int(bool(by_need_full)), _stream(stream)))


def rk_decode_step_batched(geom: Geom, sched: _Schedule, t: int, layers, q_ptrs, out_ptrs, seq_lens, max_len: int,
                           max_recent: int, ws_ptrs, workspace_bytes: int, stream=None) -> str:
    """rk_decode_step with one workspace per layer and the refreshes of a full step batched."""
    rc = lib.rk_decode_step_batched(C.byref(geom.c()), C.byref(sched), int(t), len(layers), layers, q_ptrs, out_ptrs,
                                    _dev(seq_lens, torch.int32, "seq_lens", (geom.batch,)), int(max_len), int(max_recent),
                                    ws_ptrs, int(workspace_bytes), _stream(stream))
    if rc <= 0:
        _check("rk_decode_step_batched", rc if rc < 0 else -1)
    return STEP_KINDS[rc]
