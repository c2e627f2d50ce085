"""ctypes front end of the CPU oracle (oracle/tamoe_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
package.  It imports nothing from the HIP package and the HIP package imports nothing from
here.  All arithmetic lives in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tamoe_oracle.c")
_SO = os.path.join(_HERE, "libtamoe_oracle.so")

F32 = 0
BF16 = 1
F16 = 2

_lib = None


def build(force: bool = True) -> str:
    """Compile the oracle with gcc.  -O2, OpenMP for the optional parallel-for over tokens;
    -ffp-contract=off so every product and sum is rounded as written."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_SO):
        build(force=True)
    lib = ctypes.CDLL(_SO)
    c_i32, c_i64, c_dbl, c_vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
    sig = {
        "orc_set_threads": (None, [c_i32]),
        "orc_max_threads": (c_i32, []),
        "orc_round_to_bf16": (ctypes.c_uint16, [c_dbl]),
        "orc_round_to_f16": (ctypes.c_uint16, [c_dbl]),
        "orc_half_value": (c_dbl, [ctypes.c_uint16]),
        "orc_smooth_beta": (c_i32, [c_vp, c_vp, c_i32, c_vp]),
        "orc_target_pattern": (None, [c_vp, c_i32, c_i32, c_i32, c_i32, c_i64, c_vp]),
        "orc_penalty": (None, [c_vp, c_i32, c_vp]),
        "orc_capacity": (None, [c_vp, c_i32, c_i32, c_i64, c_dbl, c_i32, c_vp]),
        "orc_exchange_cost": (c_dbl, [c_vp, c_vp, c_vp, c_i32, c_i32, c_dbl]),
        "orc_logits": (None, [c_vp, c_vp, c_i32, c_i64, c_i32, c_i32, c_vp]),
        "orc_softmax": (None, [c_vp, c_i64, c_i32, c_vp]),
        "orc_topk": (None, [c_vp, c_vp, c_i64, c_i32, c_i32, c_vp, c_vp]),
        "orc_counts": (None, [c_vp, c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp]),
        "orc_l_aux": (c_dbl, [c_vp, c_vp, c_i32, c_i64]),
        "orc_l_topo": (c_dbl, [c_vp, c_vp, c_vp, c_i32, c_i32, c_i64]),
        "orc_slots": (c_i64, [c_vp, c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp, c_vp, c_vp]),
        "orc_scatter": (None, [c_vp, c_i32, c_vp, c_i64, c_i32, c_i32, c_vp]),
        "orc_combine": (None, [c_vp, c_i32, c_vp, c_vp, c_i64, c_i32, c_i32, c_vp, c_vp]),
        "orc_gate_bwd": (None, [c_vp, c_vp, c_vp, c_vp, c_vp, c_dbl, c_i64, c_i32, c_i32, c_i32, c_vp]),
        "orc_combine_bwd": (None, [c_vp, c_vp, c_i32, c_vp, c_vp, c_i64, c_i64, c_i32, c_i32, c_vp, c_vp, c_vp]),
        "orc_dispatch_bwd": (None, [c_vp, c_i32, c_vp, c_i64, c_i32, c_i32, c_vp, c_vp]),
        "orc_penalty_softmax": (None, [c_vp, c_i32, c_dbl, c_vp]),
        "orc_renorm_topk": (None, [c_vp, c_i64, c_i32, c_vp]),
        "orc_renorm_topk_bwd": (None, [c_vp, c_vp, c_i64, c_i32, c_vp]),
        "orc_slots_padded": (None, [c_vp, c_vp, c_i64, c_i32, c_i32, c_i32, c_vp, c_vp]),
        "orc_minmax_pattern": (c_dbl, [c_vp, c_vp, c_i32, c_i32, c_i32, c_i64, c_dbl, c_vp]),
        "orc_ring_table": (None, [c_vp, c_vp, c_i32, c_dbl, c_dbl, c_vp, c_vp, c_vp]),
        "orc_tree_levels": (c_i32, [ctypes.c_char_p, c_i32, c_i32, c_vp, ctypes.c_char_p, c_i32, c_vp]),
        "orc_regroup": (c_i64, [c_vp, c_i32, c_vp, c_i32, c_i32, c_i32, c_i32, c_vp, c_vp]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _lib = lib
    return lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def _storage(a: np.ndarray, dtype: int) -> np.ndarray:
    want = np.float32 if dtype == F32 else np.uint16
    if a.dtype != want:
        raise TypeError(f"storage dtype {dtype} needs a {want} array, got {a.dtype}")
    return np.ascontiguousarray(a)


def set_threads(n: int) -> None:
    _load().orc_set_threads(int(n))


def max_threads() -> int:
    return int(_load().orc_max_threads())


def round_to_f16(v: float) -> int:
    """Bit pattern of the half-precision value nearest to the double v (ties to even)."""
    return int(_load().orc_round_to_f16(float(v)))


def half_value(bits: int) -> float:
    """Exact value of a half-precision bit pattern."""
    return float(_load().orc_half_value(int(bits)))


def round_to_bf16(v: float) -> int:
    return int(_load().orc_round_to_bf16(float(v)))


# ---- setup ------------------------------------------------------------------

def smooth_beta(beta, level) -> np.ndarray:
    beta = _c(beta, np.float64)
    level = _c(level, np.int32)
    P = beta.shape[0]
    assert beta.shape == (P, P) and level.shape == (P, P)
    out = np.empty((P, P), dtype=np.float64)
    rc = _load().orc_smooth_beta(_p(beta), _p(level), P, _p(out))
    if rc != 0:
        raise ValueError("bad level table")
    return out


def target_pattern(beta_hat, N: int, rank: int, k: int, S: int) -> np.ndarray:
    beta_hat = _c(beta_hat, np.float64)
    P = beta_hat.shape[0]
    assert N % P == 0 and 0 <= rank < P
    out = np.empty((N,), dtype=np.float64)
    _load().orc_target_pattern(_p(beta_hat), P, N, rank, k, S, _p(out))
    return out


def penalty(c_hat) -> np.ndarray:
    c_hat = _c(c_hat, np.float64)
    out = np.empty_like(c_hat)
    _load().orc_penalty(_p(c_hat), c_hat.shape[0], _p(out))
    return out


def penalty_softmax(c_hat, tau: float) -> np.ndarray:
    c_hat = _c(c_hat, np.float64)
    out = np.empty_like(c_hat)
    _load().orc_penalty_softmax(_p(c_hat), c_hat.shape[0], float(tau), _p(out))
    return out


def minmax_pattern(alpha_row, beta_row, N: int, k: int, S: int, bytes_per_row: float):
    """Row problem with the latency kept -> (c_hat[N], completion time T)."""
    beta_row = _c(beta_row, np.float64)
    alpha_row = None if alpha_row is None else _c(alpha_row, np.float64)
    P = beta_row.shape[0]
    assert N % P == 0
    out = np.empty((N,), dtype=np.float64)
    T = _load().orc_minmax_pattern(_p(alpha_row), _p(beta_row), P, N, k, S, float(bytes_per_row), _p(out))
    return out, float(T)


def ring_table(beta_link, alpha_link=None, self_beta: float = 1.0, self_alpha: float = 0.0):
    """-> (beta[P,P], alpha[P,P], level[P,P]) of a ring whose link q joins devices q and q+1."""
    beta_link = _c(beta_link, np.float64)
    alpha_link = None if alpha_link is None else _c(alpha_link, np.float64)
    P = beta_link.shape[0]
    beta = np.empty((P, P), dtype=np.float64)
    alpha = np.empty((P, P), dtype=np.float64)
    level = np.empty((P, P), dtype=np.int32)
    _load().orc_ring_table(_p(beta_link), _p(alpha_link), P, float(self_beta), float(self_alpha), _p(beta), _p(alpha),
                           _p(level))
    return beta, alpha, level


def tree_levels(text: str, merge: bool, max_P: int = 1024, want_order: bool = False):
    """Nested-list tree -> (level[P,P] in the device numbers of the tree as given, notation of the
    labelled tree[, device numbers in the order in which that tree lists them]).  Raises ValueError on
    bad text."""
    level = np.empty((max_P * max_P,), dtype=np.int32)
    order = np.empty((max_P,), dtype=np.int32)
    buf = ctypes.create_string_buffer(4096)
    P = _load().orc_tree_levels(text.encode(), 1 if merge else 0, max_P, _p(level), buf, 4096, _p(order))
    if P < 0:
        raise ValueError(f"orc_tree_levels({text!r}) failed with {P}")
    out = (level[:P * P].reshape(P, P).copy(), buf.value.decode())
    return out + (order[:P].copy(),) if want_order else out


def capacity(c_hat, k: int, S: int, cf: float, mode: int) -> np.ndarray:
    c_hat = _c(c_hat, np.float64)
    out = np.empty((c_hat.shape[0],), dtype=np.int32)
    _load().orc_capacity(_p(c_hat), c_hat.shape[0], k, S, float(cf), mode, _p(out))
    return out


def exchange_cost(alpha, beta, c, bytes_per_row: float) -> float:
    beta = _c(beta, np.float64)
    c = _c(c, np.float64)
    P = beta.shape[0]
    N = c.shape[1]
    assert c.shape[0] == P and N % P == 0
    alpha = None if alpha is None else _c(alpha, np.float64)
    return float(_load().orc_exchange_cost(_p(alpha), _p(beta), _p(c), P, N, float(bytes_per_row)))


# ---- gate -------------------------------------------------------------------

def logits(x, w, dtype: int) -> np.ndarray:
    x = _storage(x, dtype)
    w = _storage(w, dtype)
    S, d = x.shape
    N = w.shape[0]
    assert w.shape[1] == d
    out = np.empty((S, N), dtype=np.float64)
    _load().orc_logits(_p(x), _p(w), dtype, S, d, N, _p(out))
    return out


def softmax(lg) -> np.ndarray:
    lg = _c(lg, np.float64)
    S, N = lg.shape
    out = np.empty((S, N), dtype=np.float64)
    _load().orc_softmax(_p(lg), S, N, _p(out))
    return out


def topk(lg, G, k: int):
    lg = _c(lg, np.float64)
    G = _c(G, np.float64)
    S, N = lg.shape
    assert 1 <= k <= N
    idx = np.empty((S, k), dtype=np.int32)
    wgt = np.empty((S, k), dtype=np.float64)
    _load().orc_topk(_p(lg), _p(G), S, N, k, _p(idx), _p(wgt))
    return idx, wgt


def counts(idx, G, P: int):
    idx = _c(idx, np.int32)
    G = _c(G, np.float64)
    S, k = idx.shape
    N = G.shape[1]
    assert N % P == 0
    c_e = np.empty((N,), dtype=np.int32)
    c_d = np.empty((P,), dtype=np.int32)
    m = np.empty((N,), dtype=np.float64)
    _load().orc_counts(_p(idx), _p(G), S, N, P, k, _p(c_e), _p(c_d), _p(m))
    return c_e, c_d, m


def l_aux(m, c, S: int) -> float:
    m = _c(m, np.float64)
    c = _c(c, np.int32)
    return float(_load().orc_l_aux(_p(m), _p(c), m.shape[0], S))


def l_topo(p, m, c, P: int, S: int) -> float:
    p = _c(p, np.float64)
    m = _c(m, np.float64)
    c = _c(c, np.int32)
    return float(_load().orc_l_topo(_p(p), _p(m), _p(c), m.shape[0], P, S))


# ---- dispatch / combine -----------------------------------------------------

def slots(idx, cap, P: int):
    idx = _c(idx, np.int32)
    cap = _c(cap, np.int32)
    S, k = idx.shape
    N = cap.shape[0]
    assert N % P == 0
    slot = np.empty((S, k), dtype=np.int32)
    kept = np.empty((N,), dtype=np.int32)
    off = np.empty((N + 1,), dtype=np.int32)
    scd = np.empty((P,), dtype=np.int32)
    K = _load().orc_slots(_p(idx), _p(cap), S, N, P, k, _p(slot), _p(kept), _p(off), _p(scd))
    return slot, kept, off, scd, int(K)


def slots_padded(idx, cap, N: int, C: int):
    """Fixed-size layout: slot = e*C + pos (or -1), kept[e].  cap may be None."""
    idx = _c(idx, np.int32)
    S, k = idx.shape
    cap = None if cap is None else _c(cap, np.int32)
    slot = np.empty((S, k), dtype=np.int32)
    kept = np.empty((N,), dtype=np.int32)
    _load().orc_slots_padded(_p(idx), _p(cap), S, N, k, C, _p(slot), _p(kept))
    return slot, kept


def renorm_topk(wgt) -> np.ndarray:
    wgt = _c(wgt, np.float64)
    S, k = wgt.shape
    out = np.empty_like(wgt)
    _load().orc_renorm_topk(_p(wgt), S, k, _p(out))
    return out


def renorm_topk_bwd(wgt, d_out) -> np.ndarray:
    wgt = _c(wgt, np.float64)
    d_out = _c(d_out, np.float64)
    S, k = wgt.shape
    out = np.empty_like(wgt)
    _load().orc_renorm_topk_bwd(_p(wgt), _p(d_out), S, k, _p(out))
    return out


def scatter(x, dtype: int, slot, K: int) -> np.ndarray:
    x = _storage(x, dtype)
    slot = _c(slot, np.int32)
    S, d = x.shape
    k = slot.shape[1]
    send = np.zeros((K, d), dtype=x.dtype)
    _load().orc_scatter(_p(x), dtype, _p(slot), S, d, k, _p(send))
    return send


def combine(recv, dtype: int, slot, wgt, want_exact: bool = True, want_rounded: bool = True):
    recv = _storage(recv, dtype)
    slot = _c(slot, np.int32)
    wgt = _c(wgt, np.float64)
    S, k = slot.shape
    d = recv.shape[1]
    y_exact = np.empty((S, d), dtype=np.float64) if want_exact else None
    y = np.empty((S, d), dtype=recv.dtype) if want_rounded else None
    _load().orc_combine(_p(recv), dtype, _p(slot), _p(wgt), S, d, k, _p(y_exact), _p(y))
    return y_exact, y


# ---- backward -----------------------------------------------------------------

def gate_bwd(lg, idx, dwgt, p, c, loss_scale: float, P: int) -> np.ndarray:
    lg = _c(lg, np.float64)
    idx = _c(idx, np.int32)
    dwgt = _c(dwgt, np.float64)
    c = _c(c, np.int32)
    p = None if p is None else _c(p, np.float64)
    S, N = lg.shape
    k = idx.shape[1]
    out = np.empty((S, N), dtype=np.float64)
    _load().orc_gate_bwd(_p(lg), _p(idx), _p(dwgt), _p(p), _p(c), float(loss_scale), S, N, P, k, _p(out))
    return out


def combine_bwd(dy, recv, dtype: int, slot, wgt, want_rounded: bool = True):
    dy = _storage(dy, dtype)
    recv = _storage(recv, dtype)
    slot = _c(slot, np.int32)
    wgt = _c(wgt, np.float64)
    S, k = slot.shape
    K, d = recv.shape
    assert dy.shape == (S, d)
    drecv_exact = np.empty((K, d), dtype=np.float64)
    drecv = np.empty((K, d), dtype=recv.dtype) if want_rounded else None
    dwgt = np.empty((S, k), dtype=np.float64)
    _load().orc_combine_bwd(_p(dy), _p(recv), dtype, _p(slot), _p(wgt), S, K, d, k, _p(drecv_exact), _p(drecv),
                            _p(dwgt))
    return drecv_exact, drecv, dwgt


def dispatch_bwd(dsend, dtype: int, slot, want_rounded: bool = True):
    dsend = _storage(dsend, dtype)
    slot = _c(slot, np.int32)
    S, k = slot.shape
    d = dsend.shape[1]
    dx_exact = np.empty((S, d), dtype=np.float64)
    dx = np.empty((S, d), dtype=dsend.dtype) if want_rounded else None
    _load().orc_dispatch_bwd(_p(dsend), dtype, _p(slot), S, d, k, _p(dx_exact), _p(dx))
    return dx_exact, dx


# ---- receive side ---------------------------------------------------------------

def regroup(rows_in, dtype: int, cnt, to_expert_major: bool):
    """cnt [P,E]: rows from source s for local expert e.  Returns (rows_out, expert_offset[E+1])."""
    rows_in = _storage(rows_in, dtype)
    cnt = _c(cnt, np.int32)
    P, E = cnt.shape
    R, d = rows_in.shape
    assert int(cnt.sum()) == R
    out = np.zeros_like(rows_in)
    eoff = np.empty((E + 1,), dtype=np.int32)
    got = _load().orc_regroup(_p(rows_in), dtype, _p(cnt), P, E, d, 1 if to_expert_major else 0, _p(out), _p(eoff))
    assert got == R
    return out, eoff


# ---- whole path (the steps above, in the paper's order) -----------------------

def setup(beta, level, N: int, rank: int, k: int, S: int, cf: float, cap_mode: int):
    """Smoothing (if a level table is given) -> target pattern -> penalty -> capacity."""
    beta_hat = smooth_beta(beta, level) if level is not None else _c(beta, np.float64)
    c_hat = target_pattern(beta_hat, N, rank, k, S)
    return c_hat, penalty(c_hat), capacity(c_hat, k, S, cf, cap_mode)


def route_from_logits(lg, k: int, P: int, p, cap):
    """softmax -> top-k -> counts -> losses -> slots on given scores."""
    lg = _c(lg, np.float64)
    S = lg.shape[0]
    G = softmax(lg)
    idx, wgt = topk(lg, G, k)
    c_e, c_d, m = counts(idx, G, P)
    slot, kept, off, scd, K = slots(idx, cap, P)
    return {
        "G": G, "topk_idx": idx, "topk_w": wgt, "c_expert": c_e, "c_device": c_d, "m": m,
        "l_aux": l_aux(m, c_e, S), "l_topo": l_topo(p, m, c_e, P, S),
        "slot": slot, "kept": kept, "off": off, "send_count_dev": scd, "K": K,
    }
