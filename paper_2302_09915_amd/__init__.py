"""MI355X-native hot path of TA-MoE: thin Python binding of the C-ABI library libtamoe.so.

Every function named tamoe_* marshals its arguments and calls the C entry point of the same
name (include/tamoe.h); all arithmetic of the path runs in the HIP kernels of the library.
PyTorch is used for device memory and streams only.  There is no fallback: if the library has
not been built, importing the binding's functions raises.

The helpers without the prefix (gate, dispatch, combine, ...) only allocate the output tensors
with torch.empty and call the tamoe_* function.
"""
from __future__ import annotations

import ctypes
import os
import threading
from typing import Dict, Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtamoe.so")

F32 = 0
BF16 = 1
F16 = 2
CAP_UNIFORM = 0
CAP_PROPORTIONAL = 1
NORM_L1 = 0
NORM_SOFTMAX = 1
MAX_EXPERTS = 128
MAX_K = 8

OK, INVALID_ARG, UNSUPPORTED, WORKSPACE_TOO_SMALL, HIP_ERROR = 0, 1, 2, 3, 4

EXPORTS = (
    "tamoe_version", "tamoe_last_error", "tamoe_topo_pattern", "tamoe_workspace_bytes",
    "tamoe_gate", "tamoe_select", "tamoe_aux_loss", "tamoe_dispatch", "tamoe_combine",
    "tamoe_gate_bwd", "tamoe_combine_bwd", "tamoe_dispatch_bwd", "tamoe_regroup",
    "tamoe_tree_levels", "tamoe_ring_table", "tamoe_minmax_pattern",
    "tamoe_penalty", "tamoe_renorm_topk", "tamoe_renorm_topk_bwd", "tamoe_dispatch_padded",
    "tamoe_dispatch_static", "tamoe_gate_dispatch",
    "tamoe_trace_start", "tamoe_trace_filter", "tamoe_trace_stop", "tamoe_trace_get", "tamoe_trace_clear",
)


class TamoeError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"tamoe status {status}: {message}")
        self.status = status
        self.message = message


_lib = None
dbl_t = ctypes.c_double


_bind_state = threading.local()


class _Recorder:
    """Stands in for the library while bind() runs a binding function: notes the entry point and its
    marshalled arguments instead of calling it."""

    def __init__(self):
        self.calls = []

    def __getattr__(self, name):
        def note(*args):
            self.calls.append((name, args))
            return OK
        return note


class BoundCall:
    """One device entry point with its arguments checked and marshalled once.  For loops that call
    the library on the same buffers again and again: converting twenty tensors costs more host time
    per call than a small launch takes on the device.  The tensors are kept alive; the stream is the
    one that was current (or given) when bind() ran, so a bound call must not be used under a stream
    capture that began afterwards."""

    __slots__ = ("_fn", "_args", "_keep")

    def __init__(self, fn, args, keep):
        self._fn, self._args, self._keep = fn, args, keep

    def __call__(self) -> None:
        status = self._fn(*self._args)
        if status != OK:
            raise TamoeError(status, lib().tamoe_last_error().decode())


def bind(entry, *args, **kwargs) -> BoundCall:
    """bind(tamoe_combine, recv, K, slot, topk_w, y) -> a callable that makes exactly that call."""
    real = lib()
    rec = _Recorder()
    _bind_state.recorder = rec
    try:
        entry(*args, **kwargs)
    finally:
        _bind_state.recorder = None
    if len(rec.calls) != 1:
        raise TamoeError(INVALID_ARG, "bind() takes one of the tamoe_* device entry points")
    name, cargs = rec.calls[0]
    return BoundCall(getattr(real, name), cargs, (args, kwargs))


def lib() -> ctypes.CDLL:
    """The loaded library.  Raises if it has not been built (python -m paper_2302_09915_amd.build)."""
    global _lib
    rec = getattr(_bind_state, "recorder", None)
    if rec is not None:
        return rec
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_09915_amd.build`")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, dbl, vp, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_size_t
    L.tamoe_version.restype = i32
    L.tamoe_version.argtypes = []
    L.tamoe_last_error.restype = ctypes.c_char_p
    L.tamoe_last_error.argtypes = []
    L.tamoe_topo_pattern.restype = i32
    L.tamoe_topo_pattern.argtypes = [vp, vp, i32, i32, i32, i32, i64, dbl, i32, vp, vp, vp]
    L.tamoe_workspace_bytes.restype = sz
    L.tamoe_workspace_bytes.argtypes = [i64, i32, i32, i32, i32, i32]
    L.tamoe_gate.restype = i32
    L.tamoe_gate.argtypes = [vp, vp, i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tamoe_select.restype = i32
    L.tamoe_select.argtypes = [vp, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tamoe_aux_loss.restype = i32
    L.tamoe_aux_loss.argtypes = [vp, vp, vp, i32, i32, i64, vp, vp]
    L.tamoe_dispatch.restype = i32
    L.tamoe_dispatch.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp]
    L.tamoe_gate_dispatch.restype = i32
    L.tamoe_gate_dispatch.argtypes = [vp, vp, i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                      vp, vp, vp, vp, vp, vp, sz, vp]
    L.tamoe_dispatch_static.restype = i32
    L.tamoe_dispatch_static.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp]
    L.tamoe_combine.restype = i32
    L.tamoe_combine.argtypes = [vp, i64, vp, vp, i32, i64, i32, i32, vp, vp]
    L.tamoe_gate_bwd.restype = i32
    L.tamoe_gate_bwd.argtypes = [vp, vp, vp, vp, vp, ctypes.c_float, i64, i32, i32, i32, vp, vp]
    L.tamoe_combine_bwd.restype = i32
    L.tamoe_combine_bwd.argtypes = [vp, vp, i64, vp, vp, i32, i64, i32, i32, vp, vp, vp]
    L.tamoe_dispatch_bwd.restype = i32
    L.tamoe_dispatch_bwd.argtypes = [vp, i64, vp, i32, i64, i32, i32, vp, vp]
    L.tamoe_regroup.restype = i32
    L.tamoe_regroup.argtypes = [vp, vp, i32, i32, i32, i32, i64, i32, vp, vp, vp, sz, vp]
    L.tamoe_tree_levels.restype = i32
    L.tamoe_tree_levels.argtypes = [ctypes.c_char_p, i32, i32, vp, ctypes.POINTER(ctypes.c_int), ctypes.c_char_p, sz, vp]
    L.tamoe_ring_table.restype = i32
    L.tamoe_ring_table.argtypes = [vp, vp, i32, dbl, dbl, vp, vp, vp]
    L.tamoe_minmax_pattern.restype = i32
    L.tamoe_minmax_pattern.argtypes = [vp, vp, i32, i32, i32, i64, dbl, vp, ctypes.POINTER(dbl)]
    L.tamoe_penalty.restype = i32
    L.tamoe_penalty.argtypes = [vp, i32, i32, dbl, vp]
    L.tamoe_renorm_topk.restype = i32
    L.tamoe_renorm_topk.argtypes = [vp, i64, i32, vp, vp]
    L.tamoe_renorm_topk_bwd.restype = i32
    L.tamoe_renorm_topk_bwd.argtypes = [vp, vp, i64, i32, vp, vp]
    L.tamoe_dispatch_padded.restype = i32
    L.tamoe_dispatch_padded.argtypes = [vp, vp, vp, i32, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.tamoe_trace_start.restype = i32
    L.tamoe_trace_start.argtypes = [i32]
    L.tamoe_trace_filter.restype = i32
    L.tamoe_trace_filter.argtypes = [ctypes.c_char_p]
    L.tamoe_trace_stop.restype = i32
    L.tamoe_trace_stop.argtypes = []
    L.tamoe_trace_get.restype = i32
    L.tamoe_trace_get.argtypes = [i32, ctypes.c_char_p, sz, ctypes.POINTER(ctypes.c_float)]
    L.tamoe_trace_clear.restype = i32
    L.tamoe_trace_clear.argtypes = []
    _lib = L
    return L


def _check(status: int) -> None:
    if status != OK:
        raise TamoeError(status, lib().tamoe_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float16:
        return F16
    raise TamoeError(UNSUPPORTED, f"storage dtype {t.dtype} is none of float32, bfloat16, float16")


def _dev(t: Optional[torch.Tensor], dtype: Optional[torch.dtype], name: str):
    """Pointer of a contiguous device tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda:
        raise TamoeError(INVALID_ARG, f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise TamoeError(INVALID_ARG, f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TamoeError(INVALID_ARG, f"{name} must have dtype {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ws(ws: torch.Tensor):
    return _dev(ws, torch.uint8, "ws"), ws.numel()


# ---- the C entry points, one to one -------------------------------------------------------

def tamoe_version() -> int:
    return int(lib().tamoe_version())


def tamoe_last_error() -> str:
    return lib().tamoe_last_error().decode()


def tamoe_topo_pattern(beta, level, P: int, N: int, rank: int, k: int, S: int, capacity_factor: float,
                       cap_mode: int):
    """Host setup.  beta [P,P] float64, level [P,P] int32 or None -> (c_hat f64[N], penalty f32[N], cap i32[N])."""
    beta = np.ascontiguousarray(beta, dtype=np.float64)
    if beta.shape != (P, P):
        raise TamoeError(INVALID_ARG, f"beta must be [{P},{P}]")
    lv = None
    if level is not None:
        lv = np.ascontiguousarray(level, dtype=np.int32)
        if lv.shape != (P, P):
            raise TamoeError(INVALID_ARG, f"level must be [{P},{P}]")
    n = max(int(N), 0)
    c_hat = np.empty(n, dtype=np.float64)
    pen = np.empty(n, dtype=np.float32)
    cap = np.empty(n, dtype=np.int32)
    _check(lib().tamoe_topo_pattern(
        beta.ctypes.data_as(ctypes.c_void_p), None if lv is None else lv.ctypes.data_as(ctypes.c_void_p),
        P, N, rank, k, S, float(capacity_factor), cap_mode,
        c_hat.ctypes.data_as(ctypes.c_void_p), pen.ctypes.data_as(ctypes.c_void_p),
        cap.ctypes.data_as(ctypes.c_void_p)))
    return c_hat, pen, cap


def _host(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def _hp(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def tamoe_tree_levels(tree: str, merge_asymmetric: bool, max_P: int = 1024, want_order: bool = False):
    """Host.  Nested-list text -> (level i32[P,P], text of the labelled tree[, device order i32[P]])."""
    level = np.empty(max_P * max_P, dtype=np.int32)
    order = np.empty(max_P, dtype=np.int32)
    P = ctypes.c_int(0)
    buf = ctypes.create_string_buffer(max(4096, 4 * len(tree) + 16))
    _check(lib().tamoe_tree_levels(tree.encode(), 1 if merge_asymmetric else 0, max_P, _hp(level), ctypes.byref(P),
                                   buf, len(buf), _hp(order)))
    n = P.value
    out = (level[:n * n].reshape(n, n).copy(), buf.value.decode())
    return out + (order[:n].copy(),) if want_order else out


def tamoe_ring_table(beta_link, alpha_link=None, self_beta: float = 1.0, self_alpha: float = 0.0):
    """Host.  Link tables of a ring -> (beta f64[P,P], alpha f64[P,P], level i32[P,P])."""
    bl = _host(beta_link, np.float64)
    al = _host(alpha_link, np.float64)
    P = bl.shape[0]
    if al is not None and al.shape != bl.shape:
        raise TamoeError(INVALID_ARG, "alpha_link must have the shape of beta_link")
    beta = np.empty((P, P), dtype=np.float64)
    alpha = np.empty((P, P), dtype=np.float64)
    level = np.empty((P, P), dtype=np.int32)
    _check(lib().tamoe_ring_table(_hp(bl), _hp(al), P, float(self_beta), float(self_alpha), _hp(beta), _hp(alpha),
                                  _hp(level)))
    return beta, alpha, level


def tamoe_minmax_pattern(alpha_row, beta_row, N: int, k: int, S: int, bytes_per_row: float):
    """Host.  Row problem with latency -> (c_hat f64[N], optimum T)."""
    br = _host(beta_row, np.float64)
    ar = _host(alpha_row, np.float64)
    P = br.shape[0]
    if ar is not None and ar.shape != br.shape:
        raise TamoeError(INVALID_ARG, "alpha_row must have the shape of beta_row")
    c_hat = np.empty(max(int(N), 0), dtype=np.float64)
    T = dbl_t(0.0)
    _check(lib().tamoe_minmax_pattern(_hp(ar), _hp(br), P, N, k, S, float(bytes_per_row), _hp(c_hat), ctypes.byref(T)))
    return c_hat, T.value


def tamoe_penalty(c_hat, norm: int, temperature: float = 1.0) -> np.ndarray:
    """Host.  c_hat f64[N] -> penalty f32[N] with Norm `norm` (NORM_L1 / NORM_SOFTMAX)."""
    c_hat = np.ascontiguousarray(c_hat, dtype=np.float64)
    pen = np.empty(c_hat.shape[0], dtype=np.float32)
    _check(lib().tamoe_penalty(c_hat.ctypes.data_as(ctypes.c_void_p), c_hat.shape[0], norm, float(temperature),
                               pen.ctypes.data_as(ctypes.c_void_p)))
    return pen


def tamoe_workspace_bytes(S: int, d: int, N: int, P: int, k: int, dtype: int) -> int:
    return int(lib().tamoe_workspace_bytes(S, d, N, P, k, dtype))


def tamoe_gate(x, w, P: int, k: int, logits, topk_idx, topk_w, m, c_expert, c_device, ws, stream=None) -> None:
    S, d = x.shape
    N = w.shape[0]
    if w.shape[1] != d or w.dtype != x.dtype:
        raise TamoeError(INVALID_ARG, "w must be [N,d] with the dtype of x")
    wsp, wsn = _ws(ws)
    _check(lib().tamoe_gate(
        _dev(x, None, "x"), _dev(w, None, "w"), _dtype_code(x), S, d, N, P, k,
        _dev(logits, torch.float32, "logits"), _dev(topk_idx, torch.int32, "topk_idx"),
        _dev(topk_w, torch.float32, "topk_w"), _dev(m, torch.float32, "m"),
        _dev(c_expert, torch.int32, "c_expert"), _dev(c_device, torch.int32, "c_device"),
        wsp, wsn, _stream(stream)))


def tamoe_select(logits, P: int, k: int, topk_idx, topk_w, m, c_expert, c_device, ws, stream=None) -> None:
    S, N = logits.shape
    wsp, wsn = _ws(ws)
    _check(lib().tamoe_select(
        _dev(logits, torch.float32, "logits"), S, N, P, k,
        _dev(topk_idx, torch.int32, "topk_idx"), _dev(topk_w, torch.float32, "topk_w"),
        _dev(m, torch.float32, "m"), _dev(c_expert, torch.int32, "c_expert"),
        _dev(c_device, torch.int32, "c_device"), wsp, wsn, _stream(stream)))


def tamoe_aux_loss(m, c_expert, penalty, P: int, S: int, loss, stream=None) -> None:
    N = m.shape[0]
    _check(lib().tamoe_aux_loss(
        _dev(m, torch.float32, "m"), _dev(c_expert, torch.int32, "c_expert"),
        _dev(penalty, torch.float32, "penalty"), N, P, S, _dev(loss, torch.float32, "loss"), _stream(stream)))


def tamoe_dispatch(x, topk_idx, cap, N: int, P: int, send, slot, kept_expert, expert_offset, send_count_dev,
                   ws, stream=None) -> None:
    S, d = x.shape
    k = topk_idx.shape[1]
    wsp, wsn = _ws(ws)
    if send is not None and (send.dtype != x.dtype or send.numel() < S * k * d):
        raise TamoeError(INVALID_ARG, "send must have the dtype of x and room for k*S rows")
    _check(lib().tamoe_dispatch(
        _dev(x, None, "x"), _dev(topk_idx, torch.int32, "topk_idx"), _dev(cap, torch.int32, "cap"),
        _dtype_code(x), S, d, N, P, k, _dev(send, None, "send"), _dev(slot, torch.int32, "slot"),
        _dev(kept_expert, torch.int32, "kept_expert"), _dev(expert_offset, torch.int32, "expert_offset"),
        _dev(send_count_dev, torch.int32, "send_count_dev"), wsp, wsn, _stream(stream)))


def tamoe_gate_dispatch(x, w, P: int, k: int, penalty, cap, logits, topk_idx, topk_w, m, c_expert, c_device, loss,
                        send, slot, kept_expert, expert_offset, send_count_dev, ws, stream=None) -> None:
    """Gate, loss and dispatch in one call (three launches)."""
    S, d = x.shape
    N = w.shape[0]
    if w.shape[1] != d or w.dtype != x.dtype:
        raise TamoeError(INVALID_ARG, "w must be [N,d] with the dtype of x")
    if send is not None and (send.dtype != x.dtype or send.numel() < S * k * d):
        raise TamoeError(INVALID_ARG, "send must have the dtype of x and room for k*S rows")
    wsp, wsn = _ws(ws)
    _check(lib().tamoe_gate_dispatch(
        _dev(x, None, "x"), _dev(w, None, "w"), _dtype_code(x), S, d, N, P, k,
        _dev(penalty, torch.float32, "penalty"), _dev(cap, torch.int32, "cap"),
        _dev(logits, torch.float32, "logits"), _dev(topk_idx, torch.int32, "topk_idx"),
        _dev(topk_w, torch.float32, "topk_w"), _dev(m, torch.float32, "m"),
        _dev(c_expert, torch.int32, "c_expert"), _dev(c_device, torch.int32, "c_device"),
        _dev(loss, torch.float32, "loss"), _dev(send, None, "send"), _dev(slot, torch.int32, "slot"),
        _dev(kept_expert, torch.int32, "kept_expert"), _dev(expert_offset, torch.int32, "expert_offset"),
        _dev(send_count_dev, torch.int32, "send_count_dev"), wsp, wsn, _stream(stream)))


def tamoe_dispatch_static(x, topk_idx, cap, N: int, P: int, send, slot, kept_expert, expert_offset, send_count_dev,
                          stream=None) -> None:
    """tamoe_dispatch with the library's built-in scratch instead of a workspace (allocates nothing)."""
    S, d = x.shape
    k = topk_idx.shape[1]
    if send is not None and (send.dtype != x.dtype or send.numel() < S * k * d):
        raise TamoeError(INVALID_ARG, "send must have the dtype of x and room for k*S rows")
    _check(lib().tamoe_dispatch_static(
        _dev(x, None, "x"), _dev(topk_idx, torch.int32, "topk_idx"), _dev(cap, torch.int32, "cap"),
        _dtype_code(x), S, d, N, P, k, _dev(send, None, "send"), _dev(slot, torch.int32, "slot"),
        _dev(kept_expert, torch.int32, "kept_expert"), _dev(expert_offset, torch.int32, "expert_offset"),
        _dev(send_count_dev, torch.int32, "send_count_dev"), _stream(stream)))


def tamoe_dispatch_padded(x, topk_idx, cap, N: int, P: int, C: int, send, slot, kept_expert, ws, stream=None) -> None:
    """send [N*C, d]; cap may be None (the limit is C alone)."""
    S, d = x.shape
    k = topk_idx.shape[1]
    wsp, wsn = _ws(ws)
    if send is None or send.dtype != x.dtype or send.numel() != N * C * d:
        raise TamoeError(INVALID_ARG, "send must have the dtype of x and exactly N*C rows")
    _check(lib().tamoe_dispatch_padded(
        _dev(x, None, "x"), _dev(topk_idx, torch.int32, "topk_idx"), _dev(cap, torch.int32, "cap"),
        _dtype_code(x), S, d, N, P, k, C, _dev(send, None, "send"), _dev(slot, torch.int32, "slot"),
        _dev(kept_expert, torch.int32, "kept_expert"), wsp, wsn, _stream(stream)))


def tamoe_renorm_topk(topk_w, out, stream=None) -> None:
    S, k = topk_w.shape
    if out is None or out.shape != topk_w.shape:
        raise TamoeError(INVALID_ARG, "out must have the shape of topk_w")
    _check(lib().tamoe_renorm_topk(_dev(topk_w, torch.float32, "topk_w"), S, k, _dev(out, torch.float32, "out"),
                                   _stream(stream)))


def tamoe_renorm_topk_bwd(topk_w, d_out, d_topk_w, stream=None) -> None:
    S, k = topk_w.shape
    if d_out is None or d_topk_w is None or d_out.shape != topk_w.shape or d_topk_w.shape != topk_w.shape:
        raise TamoeError(INVALID_ARG, "d_out and d_topk_w must have the shape of topk_w")
    _check(lib().tamoe_renorm_topk_bwd(_dev(topk_w, torch.float32, "topk_w"), _dev(d_out, torch.float32, "d_out"),
                                       S, k, _dev(d_topk_w, torch.float32, "d_topk_w"), _stream(stream)))


def tamoe_combine(recv, K_rows: int, slot, topk_w, y, stream=None) -> None:
    S, k = slot.shape
    d = y.shape[1]
    if recv is not None and (recv.dtype != y.dtype or recv.numel() < K_rows * d):
        raise TamoeError(INVALID_ARG, "recv must have the dtype of y and hold K_rows rows")
    _check(lib().tamoe_combine(
        _dev(recv, None, "recv"), K_rows, _dev(slot, torch.int32, "slot"),
        _dev(topk_w, torch.float32, "topk_w"), _dtype_code(y), S, d, k, _dev(y, None, "y"), _stream(stream)))


def tamoe_gate_bwd(logits, topk_idx, d_topk_w, penalty, c_expert, loss_scale: float, P: int, d_logits,
                   stream=None) -> None:
    S, N = logits.shape
    k = topk_idx.shape[1]
    _check(lib().tamoe_gate_bwd(
        _dev(logits, torch.float32, "logits"), _dev(topk_idx, torch.int32, "topk_idx"),
        _dev(d_topk_w, torch.float32, "d_topk_w"), _dev(penalty, torch.float32, "penalty"),
        _dev(c_expert, torch.int32, "c_expert"), float(loss_scale), S, N, P, k,
        _dev(d_logits, torch.float32, "d_logits"), _stream(stream)))


def tamoe_combine_bwd(dy, recv, K_rows: int, slot, topk_w, d_recv, d_topk_w, stream=None) -> None:
    S, k = slot.shape
    d = dy.shape[1]
    if recv is not None and (recv.dtype != dy.dtype or recv.numel() < K_rows * d):
        raise TamoeError(INVALID_ARG, "recv must have the dtype of dy and hold K_rows rows")
    if d_recv is not None and (d_recv.dtype != dy.dtype or d_recv.numel() < K_rows * d):
        raise TamoeError(INVALID_ARG, "d_recv must have the dtype of dy and hold K_rows rows")
    _check(lib().tamoe_combine_bwd(
        _dev(dy, None, "dy"), _dev(recv, None, "recv"), K_rows, _dev(slot, torch.int32, "slot"),
        _dev(topk_w, torch.float32, "topk_w"), _dtype_code(dy), S, d, k, _dev(d_recv, None, "d_recv"),
        _dev(d_topk_w, torch.float32, "d_topk_w"), _stream(stream)))


def tamoe_dispatch_bwd(d_send, K_rows: int, slot, d_x, stream=None) -> None:
    S, k = slot.shape
    d = d_x.shape[1]
    if d_send is not None and (d_send.dtype != d_x.dtype or d_send.numel() < K_rows * d):
        raise TamoeError(INVALID_ARG, "d_send must have the dtype of d_x and hold K_rows rows")
    _check(lib().tamoe_dispatch_bwd(
        _dev(d_send, None, "d_send"), K_rows, _dev(slot, torch.int32, "slot"), _dtype_code(d_x), S, d, k,
        _dev(d_x, None, "d_x"), _stream(stream)))


def tamoe_regroup(rows_in, recv_count, to_expert_major: bool, rows_out, expert_offset, ws, stream=None) -> None:
    """recv_count [P,E] int32 (device); rows_in / rows_out [cap_rows, d]."""
    P, E = recv_count.shape
    cap_rows, d = rows_in.shape
    if rows_out.shape != rows_in.shape or rows_out.dtype != rows_in.dtype:
        raise TamoeError(INVALID_ARG, "rows_out must have the shape and dtype of rows_in")
    wsp, wsn = _ws(ws)
    _check(lib().tamoe_regroup(
        _dev(rows_in, None, "rows_in"), _dev(recv_count, torch.int32, "recv_count"), P, E, _dtype_code(rows_in), d,
        cap_rows, 1 if to_expert_major else 0, _dev(rows_out, None, "rows_out"),
        _dev(expert_offset, torch.int32, "expert_offset"), wsp, wsn, _stream(stream)))


def tamoe_trace_start(max_launches: int) -> None:
    _check(lib().tamoe_trace_start(max_launches))


def tamoe_trace_filter(kernel_name: Optional[str]) -> None:
    _check(lib().tamoe_trace_filter(None if kernel_name is None else kernel_name.encode()))


def tamoe_trace_stop() -> int:
    n = lib().tamoe_trace_stop()
    if n < 0:
        _check(-n)
    return n


def tamoe_trace_get(i: int):
    name = ctypes.create_string_buffer(64)
    ms = ctypes.c_float(0.0)
    _check(lib().tamoe_trace_get(i, name, 64, ctypes.byref(ms)))
    return name.value.decode(), float(ms.value)


def tamoe_trace_clear() -> None:
    _check(lib().tamoe_trace_clear())


# ---- allocating helpers -------------------------------------------------------------------

def workspace(S: int, d: int, N: int, P: int, k: int, dtype: int, device="cuda") -> torch.Tensor:
    return torch.empty(tamoe_workspace_bytes(S, d, N, P, k, dtype), dtype=torch.uint8, device=device)


def _select_outputs(S: int, N: int, P: int, k: int, device) -> Dict[str, torch.Tensor]:
    return {
        "topk_idx": torch.empty((S, k), dtype=torch.int32, device=device),
        "topk_w": torch.empty((S, k), dtype=torch.float32, device=device),
        "m": torch.empty((N,), dtype=torch.float32, device=device),
        "c_expert": torch.empty((N,), dtype=torch.int32, device=device),
        "c_device": torch.empty((P,), dtype=torch.int32, device=device),
    }


def gate(x, w, P: int, k: int, want_logits: bool = True, ws=None, stream=None) -> Dict[str, torch.Tensor]:
    S, d = x.shape
    N = w.shape[0]
    out = _select_outputs(S, N, P, k, x.device)
    out["logits"] = torch.empty((S, N), dtype=torch.float32, device=x.device) if want_logits else None
    if ws is None:
        ws = workspace(S, d, N, P, k, _dtype_code(x), x.device)
    tamoe_gate(x, w, P, k, out["logits"], out["topk_idx"], out["topk_w"], out["m"], out["c_expert"],
               out["c_device"], ws, stream)
    return out


def select(logits, P: int, k: int, ws=None, stream=None) -> Dict[str, torch.Tensor]:
    S, N = logits.shape
    out = _select_outputs(S, N, P, k, logits.device)
    if ws is None:
        ws = workspace(S, 4, N, P, k, F32, logits.device)
    tamoe_select(logits, P, k, out["topk_idx"], out["topk_w"], out["m"], out["c_expert"], out["c_device"], ws, stream)
    return out


def aux_loss(m, c_expert, penalty, P: int, S: int, stream=None) -> torch.Tensor:
    loss = torch.empty((1,), dtype=torch.float32, device=m.device)
    tamoe_aux_loss(m, c_expert, penalty, P, S, loss, stream)
    return loss


def dispatch(x, topk_idx, cap, N: int, P: int, ws=None, stream=None) -> Dict[str, torch.Tensor]:
    S, d = x.shape
    k = topk_idx.shape[1]
    dev = x.device
    out = {
        "send": torch.empty((S * k, d), dtype=x.dtype, device=dev),
        "slot": torch.empty((S, k), dtype=torch.int32, device=dev),
        "kept_expert": torch.empty((N,), dtype=torch.int32, device=dev),
        "expert_offset": torch.empty((N + 1,), dtype=torch.int32, device=dev),
        "send_count_dev": torch.empty((P,), dtype=torch.int32, device=dev),
    }
    if ws is None:
        ws = workspace(S, d, N, P, k, _dtype_code(x), dev)
    tamoe_dispatch(x, topk_idx, cap, N, P, out["send"], out["slot"], out["kept_expert"], out["expert_offset"],
                   out["send_count_dev"], ws, stream)
    return out


def gate_dispatch(x, w, P: int, k: int, penalty, cap, want_logits: bool = True, ws=None,
                  stream=None) -> Dict[str, torch.Tensor]:
    S, d = x.shape
    N = w.shape[0]
    dev = x.device
    out = _select_outputs(S, N, P, k, dev)
    out["logits"] = torch.empty((S, N), dtype=torch.float32, device=dev) if want_logits else None
    out.update({
        "loss": torch.empty((1,), dtype=torch.float32, device=dev),
        "send": torch.empty((S * k, d), dtype=x.dtype, device=dev),
        "slot": torch.empty((S, k), dtype=torch.int32, device=dev),
        "kept_expert": torch.empty((N,), dtype=torch.int32, device=dev),
        "expert_offset": torch.empty((N + 1,), dtype=torch.int32, device=dev),
        "send_count_dev": torch.empty((P,), dtype=torch.int32, device=dev),
    })
    if ws is None:
        ws = workspace(S, d, N, P, k, _dtype_code(x), dev)
    tamoe_gate_dispatch(x, w, P, k, penalty, cap, out["logits"], out["topk_idx"], out["topk_w"], out["m"],
                        out["c_expert"], out["c_device"], out["loss"], out["send"], out["slot"], out["kept_expert"],
                        out["expert_offset"], out["send_count_dev"], ws, stream)
    return out


def combine(recv, K_rows: int, slot, topk_w, d: Optional[int] = None, stream=None) -> torch.Tensor:
    S = slot.shape[0]
    d = recv.shape[1] if d is None else d
    y = torch.empty((S, d), dtype=recv.dtype, device=recv.device)
    tamoe_combine(recv, K_rows, slot, topk_w, y, stream)
    return y
