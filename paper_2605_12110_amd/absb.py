"""Thin Python binding of libabsb.so: same names as the C ABI, argument marshalling only.

Every step of the path runs in the library's HIP kernels; this module converts torch
tensors to device pointers, keeps the host-side arrays alive and turns status codes into
exceptions.  There is no fallback: a missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# ABSB_LIB names another build of the same library (the host-sanitizer build of tests/sanitized.py)
LIB_PATH = os.environ.get("ABSB_LIB") or os.path.join(_HERE, "libabsb.so")

F16, BF16 = 0, 1
REPR_MEAN, REPR_MINMAX = 0, 1
SELECT_GROUP, SELECT_PER_QUERY_HEAD, SELECT_GROUP_MAX = 0, 1, 2
STEP_AUTO, STEP_PIPELINED, STEP_UNITS, STEP_PER_STAGE = 0, 1, 2, 3

OK, ERR_NULL, ERR_BAD_SHAPE, ERR_BAD_BLOCK_SIZE, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, -1, -2, -3, -4, -5, -6
ERR_STATIC_WORKSPACE = -7
STATIC_WORKSPACE_BYTES = 16 << 20

EXPORTS = ("absb_plan", "absb_step_form_used", "absb_status_offset", "absb_workspace_init", "absb_build_centroids", "absb_score", "absb_topk", "absb_sparse_decode",
           "absb_decode_fused", "absb_tail_init", "absb_append_token", "absb_head_recall", "absb_assign_block_sizes", "absb_stream_read",
           "absb_strerror", "absb_decode_fused_static")


class AbsbError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


class _Layer(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("page_size", C.c_int32), ("dtype", C.c_int32), ("block_repr", C.c_int32),
                ("block_size", C.POINTER(C.c_int32)),
                ("kv_stride_page", C.c_int64), ("kv_stride_head", C.c_int64), ("kv_stride_tok", C.c_int64),
                ("sm_scale", C.c_float), ("sink_tokens", C.c_int32), ("recent_tokens", C.c_int32),
                ("selection", C.c_int32)]


class _Opts(C.Structure):
    _fields_ = [("step_form", C.c_int32), ("split_tokens", C.c_int32), ("score_chunk", C.c_int32),
                ("unit_tokens", C.c_int32), ("counters_zero", C.c_int32)]


class _Batch(C.Structure):
    _fields_ = [("batch", C.c_int32), ("pt_stride", C.c_int32),
                ("seq_lens_host", C.POINTER(C.c_int32)), ("seq_lens", C.c_void_p),
                ("page_table", C.c_void_p), ("cent_off", C.c_void_p),
                ("budget_host", C.POINTER(C.c_int32)), ("budget", C.c_void_p),
                ("cap_lens_host", C.POINTER(C.c_int32)), ("qmin", C.c_void_p), ("opts", _Opts)]


_lib = None


def load() -> C.CDLL:
    """Load libabsb.so (built in-tree by paper_2605_12110_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)")
        lib = C.CDLL(LIB_PATH)
        lib.absb_strerror.restype = C.c_char_p
        lib.absb_strerror.argtypes = [C.c_int]
        for name in EXPORTS:
            getattr(lib, name)            # fail loudly on a stale library
        _lib = lib
    return _lib


def strerror(status: int) -> str:
    return load().absb_strerror(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != OK:
        raise AbsbError(status, where)


def _ptr(t) -> Optional[C.c_void_p]:
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        return C.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return C.c_void_p(stream)
    return C.c_void_p(stream.cuda_stream)


def _i32_host(a: Optional[Sequence[int]]):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(a), dtype=np.int32)
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


@dataclass
class Layer:
    """Host description of a layer (mirrors absb_layer)."""
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    dtype: int
    block_size: Sequence[int]
    kv_strides: Sequence[int]          # (page, head, token) in elements
    sm_scale: float = 0.0
    block_repr: int = REPR_MEAN
    sink_tokens: int = 0
    recent_tokens: int = 0
    selection: int = SELECT_GROUP

    def __setattr__(self, name, value):
        object.__setattr__(self, name, value)
        if not name.startswith("_"):
            object.__setattr__(self, "_c", None)       # any field change invalidates the cached C struct

    def c(self) -> _Layer:
        """The absb_layer record (built once per set of field values: marshalling stays off the hot path)."""
        if getattr(self, "_c", None) is None:
            self._bs, bs_p = _i32_host(self.block_size)
            sp, sh, st = (int(x) for x in self.kv_strides)
            self._c = _Layer(self.num_q_heads, self.num_kv_heads, self.head_dim, self.page_size, self.dtype,
                             int(self.block_repr),
                             bs_p, sp, sh, st, float(self.sm_scale), int(self.sink_tokens),
                             int(self.recent_tokens), int(self.selection))
        return self._c


@dataclass
class LaunchOpts:
    """How a call is enqueued (mirrors absb_launch_opts): all zero = the library's choices."""
    step_form: int = STEP_AUTO
    split_tokens: int = 0
    score_chunk: int = 0
    unit_tokens: int = 0
    counters_zero: int = 0


@dataclass
class Batch:
    """One decode step's batch (mirrors absb_batch).  Host arrays are numpy/sequences, device
    arrays are int32 torch tensors on the GPU (or None where an entry point does not need them)."""
    seq_lens_host: Sequence[int]
    budget_host: Optional[Sequence[int]] = None
    seq_lens: object = None
    page_table: object = None
    cent_off: object = None
    budget: object = None
    pt_stride: Optional[int] = None
    cap_lens_host: Optional[Sequence[int]] = None
    qmin: object = None
    opts: LaunchOpts = None

    def __post_init__(self):
        if self.opts is None:
            self.opts = LaunchOpts()

    def __setattr__(self, name, value):
        object.__setattr__(self, name, value)
        if not name.startswith("_"):
            object.__setattr__(self, "_c", None)

    def c(self) -> _Batch:
        """The absb_batch record (cached until a field is reassigned; the tensors must stay alive)."""
        if getattr(self, "_c", None) is None:
            self._sl, sl_p = _i32_host(self.seq_lens_host)
            self._bg, bg_p = _i32_host(self.budget_host)
            pts = self.pt_stride
            if pts is None:
                pts = int(self.page_table.shape[1]) if self.page_table is not None else 0
            self._cl, cl_p = _i32_host(self.cap_lens_host)
            self._c = _Batch(len(self._sl), int(pts), sl_p, _ptr(self.seq_lens), _ptr(self.page_table),
                             _ptr(self.cent_off), bg_p, _ptr(self.budget), cl_p, _ptr(self.qmin), _Opts())
        o = self.opts                   # the options object may have been changed in place: copied every time
        self._c.opts = _Opts(int(o.step_form), int(o.split_tokens), int(o.score_chunk), int(o.unit_tokens),
                             int(o.counters_zero))
        return self._c


@dataclass
class PlanResult:
    cent_off: np.ndarray       # int32 [Bt*Hkv+1]
    total_centroids: int
    sel_stride: int
    workspace_bytes: int


def absb_plan(layer: Layer, batch: Batch) -> PlanResult:
    cl, cb = layer.c(), batch.c()
    nseg = cb.batch * layer.num_kv_heads
    off = np.zeros(max(nseg, 0) + 1, dtype=np.int32)
    total, stride, ws = C.c_int64(0), C.c_int32(0), C.c_size_t(0)
    _check(load().absb_plan(C.byref(cl), C.byref(cb), off.ctypes.data_as(C.POINTER(C.c_int32)),
                            C.byref(total), C.byref(stride), C.byref(ws)), "absb_plan")
    return PlanResult(off, int(total.value), int(stride.value), int(ws.value))


def absb_build_centroids(layer: Layer, batch: Batch, k_cache, codes, qscale, qmin, workspace, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_build_centroids(C.byref(cl), C.byref(cb), _ptr(k_cache), _ptr(codes), _ptr(qscale),
                                       _ptr(qmin), _ptr(workspace), C.c_size_t(_nbytes(workspace)),
                                       _stream(stream)), "absb_build_centroids")


def absb_score(layer: Layer, batch: Batch, q, codes, qscale, scores, score_exp=None, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_score(C.byref(cl), C.byref(cb), _ptr(q), _ptr(codes), _ptr(qscale), _ptr(scores),
                             _ptr(score_exp), _stream(stream)), "absb_score")


def absb_topk(layer: Layer, batch: Batch, scores, sel_idx, sel_cnt, sel_stride: int, workspace=None,
              stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_topk(C.byref(cl), C.byref(cb), _ptr(scores), _ptr(sel_idx), _ptr(sel_cnt),
                            C.c_int32(sel_stride), _ptr(workspace), C.c_size_t(_nbytes(workspace)),
                            _stream(stream)), "absb_topk")


def absb_sparse_decode(layer: Layer, batch: Batch, q, k_cache, v_cache, sel_idx, sel_cnt, sel_stride: int,
                       out, lse, workspace, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_sparse_decode(C.byref(cl), C.byref(cb), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                     _ptr(sel_idx), _ptr(sel_cnt), C.c_int32(sel_stride), _ptr(out), _ptr(lse),
                                     _ptr(workspace), C.c_size_t(_nbytes(workspace)), _stream(stream)),
           "absb_sparse_decode")


def absb_decode_fused(layer: Layer, batch: Batch, q, codes, qscale, k_cache, v_cache, out, lse=None,
                      sel_idx_out=None, sel_cnt_out=None, workspace=None, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_decode_fused(C.byref(cl), C.byref(cb), _ptr(q), _ptr(codes), _ptr(qscale), _ptr(k_cache),
                                    _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(sel_idx_out), _ptr(sel_cnt_out),
                                    _ptr(workspace), C.c_size_t(_nbytes(workspace)), _stream(stream)),
           "absb_decode_fused")


def absb_decode_fused_static(layer: Layer, batch: Batch, q, codes, qscale, k_cache, v_cache, out, lse=None,
                             sel_idx_out=None, sel_cnt_out=None, stream=None) -> None:
    """The step on the library's built-in scratch array: no workspace argument, nothing allocated."""
    cl, cb = layer.c(), batch.c()
    _check(load().absb_decode_fused_static(C.byref(cl), C.byref(cb), _ptr(q), _ptr(codes), _ptr(qscale),
                                           _ptr(k_cache), _ptr(v_cache), _ptr(out), _ptr(lse), _ptr(sel_idx_out),
                                           _ptr(sel_cnt_out), _stream(stream)), "absb_decode_fused_static")


def absb_step_form_used(layer: Layer, batch: Batch) -> int:
    """The absb_step_form absb_decode_fused will use for this (layer, batch, batch.opts): 1, 2 or 3."""
    cl, cb = layer.c(), batch.c()
    n = load().absb_step_form_used(C.byref(cl), C.byref(cb))
    if n < 0:
        raise AbsbError(n, "absb_step_form_used")
    return int(n)


def absb_status_offset(layer: Layer, batch: Batch) -> int:
    cl, cb = layer.c(), batch.c()
    off = C.c_size_t(0)
    _check(load().absb_status_offset(C.byref(cl), C.byref(cb), C.byref(off)), "absb_status_offset")
    return int(off.value)


def absb_workspace_init(layer: Layer, batch: Batch, workspace, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_workspace_init(C.byref(cl), C.byref(cb), _ptr(workspace), C.c_size_t(_nbytes(workspace)),
                                      _stream(stream)), "absb_workspace_init")


def absb_tail_init(layer: Layer, batch: Batch, k_cache, tail, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_tail_init(C.byref(cl), C.byref(cb), _ptr(k_cache), _ptr(tail), _stream(stream)),
           "absb_tail_init")


def absb_append_token(layer: Layer, batch: Batch, k_cache, codes, qscale, qmin, tail, clamped=None,
                      stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_append_token(C.byref(cl), C.byref(cb), _ptr(k_cache), _ptr(codes), _ptr(qscale), _ptr(qmin),
                                    _ptr(tail), _ptr(clamped), _stream(stream)), "absb_append_token")


def absb_head_recall(layer: Layer, batch: Batch, lse_selected, lse_dense, recall, stream=None) -> None:
    cl, cb = layer.c(), batch.c()
    _check(load().absb_head_recall(C.byref(cl), C.byref(cb), _ptr(lse_selected), _ptr(lse_dense), _ptr(recall),
                                   _stream(stream)), "absb_head_recall")


def absb_assign_block_sizes(recall: np.ndarray, candidates: Sequence[int], tau: float):
    """recall [n_samples, n_heads, n_cand] f32 (host) -> (block size per head, mean recall [heads, cands])."""
    rec = np.ascontiguousarray(recall, dtype=np.float32)
    n, nh, nc = rec.shape
    cand = np.ascontiguousarray(candidates, dtype=np.int32)
    out = np.empty(nh, np.int32)
    mean = np.empty((nh, nc), np.float64)
    _check(load().absb_assign_block_sizes(C.c_int32(n), C.c_int32(nh), C.c_int32(nc),
                                          rec.ctypes.data_as(C.c_void_p), cand.ctypes.data_as(C.c_void_p),
                                          C.c_double(tau), out.ctypes.data_as(C.c_void_p),
                                          mean.ctypes.data_as(C.c_void_p)), "absb_assign_block_sizes")
    return out, mean


def absb_stream_read(src, sink, stream=None) -> None:
    _check(load().absb_stream_read(_ptr(src), C.c_size_t(_nbytes(src)), _ptr(sink), _stream(stream)),
           "absb_stream_read")


def _nbytes(t) -> int:
    if t is None:
        return 0
    return int(t.numel() * t.element_size())
