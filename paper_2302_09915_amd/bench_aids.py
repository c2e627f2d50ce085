"""Binding of libtamoe_bench.so: the yardstick kernels that bench.py times beside the kernels of the
path (a plain copy, and the bare memory operations of the scatter and of the combine).  They are not
part of the product library and hold none of the method's logic."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtamoe_bench.so")
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_09915_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
        L.tamoe_copy_probe.restype = i32
        L.tamoe_copy_probe.argtypes = [vp, vp, sz, vp]
        L.tamoe_mix_probe.restype = i32
        L.tamoe_mix_probe.argtypes = [vp, vp, vp, vp, i64, i64, i32, i32, vp]
        _lib = L
    return _lib


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t: torch.Tensor, name: str) -> ctypes.c_void_p:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


def copy_probe(src: torch.Tensor, dst: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < nbytes:
        raise ValueError("dst is smaller than src")
    rc = lib().tamoe_copy_probe(_ptr(src, "src"), _ptr(dst, "dst"), nbytes, _stream(stream))
    if rc != 0:
        raise RuntimeError(f"tamoe_copy_probe failed with {rc}")


def mix_probe(a: torch.Tensor, b: torch.Tensor, row0: torch.Tensor, row1: torch.Tensor, mode: int, stream=None) -> None:
    """mode 1: b[row0[t]] = b[row1[t]] = a[t]; mode 2: b[t] = a[row0[t]] ^ a[row1[t]].  a, b: [rows, d] matrices."""
    rows = row0.shape[0]
    if row0.dtype != torch.int32 or row1.dtype != torch.int32 or row1.shape[0] != rows:
        raise ValueError("row0 and row1 must be int32 vectors of one length")
    if mode == 1:
        row_bytes, other, need = a.shape[1] * a.element_size(), b.shape[0], a.shape[0]
    else:
        row_bytes, other, need = b.shape[1] * b.element_size(), a.shape[0], b.shape[0]
    if need < rows:
        raise ValueError("the matrix walked in order has fewer rows than the row tables")
    if a.shape[1] * a.element_size() != b.shape[1] * b.element_size():
        raise ValueError("a and b must have rows of the same length")
    rc = lib().tamoe_mix_probe(_ptr(a, "a"), _ptr(b, "b"), _ptr(row0, "row0"), _ptr(row1, "row1"), rows, other,
                               row_bytes, mode, _stream(stream))
    if rc != 0:
        raise RuntimeError(f"tamoe_mix_probe failed with {rc}")
