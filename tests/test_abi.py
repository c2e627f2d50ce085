"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, rejects bad
arguments with the documented status codes before touching a GPU, and its host-side setup
function agrees with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import tamoe_workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    import paper_2302_09915_amd as T

    if not os.path.exists(T.LIB_PATH):
        from paper_2302_09915_amd import build

        build.build()
    T.lib()
    return T


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "tamoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tamoe_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(T):
    names = _declared_symbols()
    assert set(names) == set(T.EXPORTS), names
    L = ctypes.CDLL(T.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None
    assert T.tamoe_version() == 1


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 and as C++ with no torch or HIP types,
    and a C program must link against the library through it."""
    import shutil
    import subprocess

    hdr = os.path.join(ROOT, "include", "tamoe.h")
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "c++")):
        if shutil.which(cc) is None:
            pytest.skip(f"{cc} not found")
        subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", lang, hdr], check=True)
    text = open(hdr).read()
    assert "#include <hip" not in text and "torch" not in text
    src = tmp_path / "use.c"
    src.write_text('#include "tamoe.h"\n#include <stdio.h>\n'
                   'int main(void) { double c[2] = {1.0, 3.0}; float p[2];\n'
                   '  if (tamoe_version() != TAMOE_VERSION) return 1;\n'
                   '  if (tamoe_penalty(c, 2, TAMOE_NORM_L1, 0.0, p) != TAMOE_OK) return 2;\n'
                   '  if (tamoe_penalty(c, 0, TAMOE_NORM_L1, 0.0, p) != TAMOE_INVALID_ARG) return 3;\n'
                   '  printf("%.2f %.2f %s\\n", p[0], p[1], tamoe_last_error()); return 0; }\n')
    import paper_2302_09915_amd as pkg
    libdir = os.path.dirname(pkg.LIB_PATH)
    exe = tmp_path / "use"
    r = subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-L", libdir, "-ltamoe",
                        f"-Wl,-rpath,{libdir}", "-o", str(exe)], capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("cannot link a C program against libtamoe here: " + r.stderr[-300:])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stderr
    assert out.stdout.startswith("0.75 0.25 tamoe_penalty")


def test_limits_match_header(T):
    text = open(os.path.join(ROOT, "include", "tamoe.h")).read()
    assert int(re.search(r"#define TAMOE_MAX_EXPERTS (\d+)", text).group(1)) == T.MAX_EXPERTS
    assert int(re.search(r"#define TAMOE_MAX_K (\d+)", text).group(1)) == T.MAX_K


# ---- host setup function against the oracle -------------------------------------------------
@pytest.mark.parametrize("name", list(W.WORKLOADS))
@pytest.mark.parametrize("cap_mode", [0, 1])
def test_topo_pattern_matches_oracle(T, oracle, name, cap_mode):
    wl = W.WORKLOADS[name]
    beta, level = W.topology(wl)
    for rank in (0, wl.P // 2 + 1, wl.P - 1):
        c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, rank, wl.k, wl.S, wl.capacity_factor, cap_mode)
        oc, op, ocap = oracle.setup(beta, level, wl.N, rank, wl.k, wl.S, wl.capacity_factor, cap_mode)
        np.testing.assert_allclose(c_hat, oc, rtol=1e-13)
        np.testing.assert_allclose(pen, op, rtol=1e-6)           # float output
        np.testing.assert_array_equal(cap, ocap)


def test_topo_pattern_smooths_noisy_tables_like_the_oracle(T, oracle):
    noisy, level = W.noisy_topology(4, 4, 8.0, seed=21)
    level = level.copy()
    np.fill_diagonal(level, 2)                      # self transfers on a level of their own
    noisy[np.diag_indices(16)] *= 0.1
    for rank in (0, 9):
        c_hat, pen, cap = T.tamoe_topo_pattern(noisy, level, 16, 32, rank, 2, 4096, 1.25, 1)
        oc, op, ocap = oracle.setup(noisy, level, 32, rank, 2, 4096, 1.25, 1)
        np.testing.assert_allclose(c_hat, oc, rtol=1e-12)
        np.testing.assert_allclose(pen, op, rtol=1e-6)
        np.testing.assert_array_equal(cap, ocap)
    # labels are names, not sizes: huge ones cost nothing and give the same pattern
    big = np.where(level == 0, 7, np.where(level == 1, 2_000_000_000, 1_999_999_999)).astype(np.int32)
    c_big, _, _ = T.tamoe_topo_pattern(noisy, big, 16, 32, 9, 2, 4096, 1.25, 1)
    np.testing.assert_allclose(c_big, oc, rtol=1e-12)
    # without a level table the raw row is used
    c_hat, _, _ = T.tamoe_topo_pattern(noisy, None, 16, 16, 3, 1, 1000, 1.0, 0)
    np.testing.assert_allclose(c_hat, oracle.target_pattern(noisy, 16, 3, 1, 1000), rtol=1e-13)


def test_topo_pattern_rejects_bad_arguments(T):
    beta, level = W.two_tier_topology(2, 2, 4.0)
    ok = dict(beta=beta, level=level, P=4, N=8, rank=0, k=2, S=100, capacity_factor=1.0, cap_mode=0)

    def call(**kw):
        a = dict(ok, **kw)
        return T.tamoe_topo_pattern(a["beta"], a["level"], a["P"], a["N"], a["rank"], a["k"], a["S"],
                                    a["capacity_factor"], a["cap_mode"])

    call()
    for bad in (dict(rank=4), dict(rank=-1), dict(N=6), dict(k=9), dict(S=0), dict(cap_mode=5),
                dict(capacity_factor=0.0), dict(capacity_factor=float("nan"))):
        with pytest.raises(T.TamoeError) as ei:
            call(**bad)
        assert ei.value.status == T.INVALID_ARG, bad
        assert "tamoe_topo_pattern" in ei.value.message
    b2 = beta.copy(); b2[1, 2] = 0.0
    with pytest.raises(T.TamoeError):
        call(beta=b2)
    b3 = beta.copy(); b3[0, 0] = float("inf")
    with pytest.raises(T.TamoeError):
        call(beta=b3)
    l2 = level.copy(); l2[0, 1] = -1
    with pytest.raises(T.TamoeError):
        call(level=l2)


def test_penalty_norms_match_oracle(T, oracle):
    for name, wl in W.WORKLOADS.items():
        beta, level = W.topology(wl)
        c_hat, pen, _ = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor, 0)
        np.testing.assert_array_equal(T.tamoe_penalty(c_hat, T.NORM_L1), pen)
        for tau in (0.0, 0.5, 2.0, 6.0):
            got = T.tamoe_penalty(c_hat, T.NORM_SOFTMAX, tau)
            ref = oracle.penalty_softmax(oracle.target_pattern(oracle.smooth_beta(beta, level), wl.N, wl.rank, wl.k,
                                                               wl.S), tau)
            assert got.dtype == np.float32
            np.testing.assert_allclose(got, ref, rtol=2e-7, atol=1e-45, err_msg=f"{name} tau={tau}")
    with pytest.raises(T.TamoeError) as ei:
        T.tamoe_penalty(np.array([1.0, 0.0]), T.NORM_SOFTMAX, 1.0)
    assert ei.value.status == T.INVALID_ARG and "c_hat[1]" in ei.value.message
    for bad in (dict(norm=3), dict(temperature=-1.0), dict(temperature=float("inf"))):
        with pytest.raises(T.TamoeError):
            T.tamoe_penalty(np.array([1.0, 2.0]), bad.get("norm", T.NORM_SOFTMAX), bad.get("temperature", 1.0))


# ---- argument checks of the device entry points (they fail before any HIP call) -------------
def test_device_entry_points_reject_bad_shapes_without_a_gpu(T):
    L = T.lib()
    one = ctypes.c_void_p(256)      # a non-null, aligned, never dereferenced address
    odd = ctypes.c_void_p(260)
    big = 1 << 30

    def status(rc, code, needle):
        assert rc == code, (rc, T.tamoe_last_error())
        assert needle in T.tamoe_last_error()

    # gate
    status(L.tamoe_gate(one, one, 1, 64, 64, 8, 4, 9, None, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "k = 9 exceeds N")
    status(L.tamoe_gate(one, one, 1, 64, 64, 6, 4, 1, None, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "not a multiple of P")
    status(L.tamoe_gate(one, one, 1, 64, 64, 256, 4, 1, None, one, one, one, one, one, one, big, None),
           T.UNSUPPORTED, "limit of 128 experts")
    status(L.tamoe_gate(one, one, 1, 64, 64, 16, 4, 12, None, one, one, one, one, one, one, big, None),
           T.UNSUPPORTED, "k = 12 exceeds the limit")
    status(L.tamoe_gate(one, one, 7, 64, 64, 8, 4, 1, None, one, one, one, one, one, one, big, None),
           T.UNSUPPORTED, "dtype 7")
    status(L.tamoe_gate(one, one, 1, 64, 60, 8, 4, 1, None, one, one, one, one, one, one, big, None),
           T.UNSUPPORTED, "multiple of 16 bytes")
    status(L.tamoe_gate(None, one, 1, 64, 64, 8, 4, 1, None, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "x is NULL")
    status(L.tamoe_gate(odd, one, 1, 64, 64, 8, 4, 1, None, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "x is not 16-byte aligned")
    status(L.tamoe_gate(one, one, 1, 64, 64, 8, 4, 1, None, one, one, one, one, one, one, 16, None),
           T.WORKSPACE_TOO_SMALL, "workspace has 16 bytes")
    status(L.tamoe_gate(one, one, 1, -1, 64, 8, 4, 1, None, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "negative")
    # select
    status(L.tamoe_select(None, 64, 8, 4, 1, one, one, one, one, one, one, big, None), T.INVALID_ARG, "logits is NULL")
    # aux loss
    status(L.tamoe_aux_loss(one, one, None, 8, 4, 0, one, None), T.INVALID_ARG, "S = 0")
    status(L.tamoe_aux_loss(one, one, None, 8, 4, 10, None, None), T.INVALID_ARG, "loss is NULL")
    # dispatch
    status(L.tamoe_dispatch(one, one, None, 1, 64, 64, 8, 4, 2, one, one, one, one, one, one, big, None),
           T.INVALID_ARG, "cap is NULL")
    status(L.tamoe_dispatch(one, one, one, 1, 64, 64, 8, 4, 2, one, one, one, one, one, one, 0, None),
           T.WORKSPACE_TOO_SMALL, "needed")
    status(L.tamoe_dispatch(one, one, one, 1, 1 << 30, 64, 8, 4, 2, one, one, one, one, one, one, big, None),
           T.UNSUPPORTED, "int32")
    # dispatch with the built-in scratch: the same checks, and the size limit before anything else happens
    status(L.tamoe_dispatch_static(one, one, None, 1, 64, 64, 8, 4, 2, one, one, one, one, one, None),
           T.INVALID_ARG, "cap is NULL")
    status(L.tamoe_dispatch_static(one, one, one, 1, 64, 64, 8, 4, 2, one, one, None, one, one, None),
           T.INVALID_ARG, "kept_expert is NULL")
    status(L.tamoe_dispatch_static(one, one, one, 1, 300 * 1024, 64, 128, 64, 8, one, one, one, one, one, None),
           T.UNSUPPORTED, "built-in scratch")
    # gate + loss + dispatch in one call
    gd = lambda **kw: L.tamoe_gate_dispatch(
        kw.get("x", one), one, kw.get("dtype", 1), kw.get("S", 64), kw.get("d", 64), kw.get("N", 8), 4, kw.get("k", 2),
        None, kw.get("cap", one), None, one, one, one, one, one, kw.get("loss", one), kw.get("send", one), one, one,
        kw.get("off", one), one, one, kw.get("ws_bytes", big), None)
    status(gd(k=9), T.INVALID_ARG, "k = 9 exceeds N")
    status(gd(N=6), T.INVALID_ARG, "not a multiple of P")
    status(gd(d=60), T.UNSUPPORTED, "multiple of 16 bytes")
    status(gd(x=None), T.INVALID_ARG, "x is NULL")
    status(gd(cap=None), T.INVALID_ARG, "cap is NULL")
    status(gd(send=None), T.INVALID_ARG, "send is NULL")
    status(gd(off=None), T.INVALID_ARG, "expert_offset is NULL")
    status(gd(loss=odd if False else ctypes.c_void_p(258)), T.INVALID_ARG, "loss is not 4-byte aligned")
    status(gd(ws_bytes=16), T.WORKSPACE_TOO_SMALL, "workspace has 16 bytes")
    status(gd(S=1 << 30), T.UNSUPPORTED, "int32")
    # combine
    status(L.tamoe_combine(one, 10, one, one, 1, 64, 64, 0, one, None), T.INVALID_ARG, "k = 0")
    status(L.tamoe_combine(one, 10, one, one, 1, 64, 64, 2, None, None), T.INVALID_ARG, "y is NULL")
    status(L.tamoe_combine(one, 10, one, one, 0, 64, 6, 2, one, None), T.UNSUPPORTED, "16 bytes")
    # backward
    status(L.tamoe_combine_bwd(one, one, 10, one, one, 1, 64, 64, 9, one, one, None), T.UNSUPPORTED, "k = 9 exceeds")
    status(L.tamoe_combine_bwd(one, one, -1, one, one, 1, 64, 64, 2, one, one, None), T.INVALID_ARG, "negative")
    status(L.tamoe_combine_bwd(one, one, 10, one, one, 1, 64, 64, 2, one, None, None), T.INVALID_ARG, "d_topk_w is NULL")
    status(L.tamoe_gate_bwd(one, one, one, None, one, 1.0, 64, 8, 3, 1, one, None), T.INVALID_ARG, "not a multiple of P")
    status(L.tamoe_gate_bwd(one, one, one, None, one, 1.0, 64, 8, 4, 1, None, None), T.INVALID_ARG, "d_logits is NULL")
    status(L.tamoe_dispatch_bwd(one, 10, one, 1, 64, 60, 2, one, None), T.UNSUPPORTED, "16 bytes")
    # regroup
    status(L.tamoe_regroup(one, one, 0, 2, 1, 64, 10, 1, one, None, one, big, None), T.INVALID_ARG, "must be positive")
    status(L.tamoe_regroup(one, one, 64, 4, 1, 64, 10, 1, one, None, one, big, None), T.UNSUPPORTED, "exceeds the limit of 128")
    status(L.tamoe_regroup(one, one, 4, 2, 1, 64, -1, 1, one, None, one, big, None), T.INVALID_ARG, "cap_rows")
    status(L.tamoe_regroup(one, one, 4, 2, 1, 64, 10, 1, one, None, one, 8, None), T.WORKSPACE_TOO_SMALL, "needed")
    status(L.tamoe_regroup(one, one, 4, 2, 1, 60, 10, 1, one, None, one, big, None), T.UNSUPPORTED, "16 bytes")
    # variants
    status(L.tamoe_renorm_topk(one, 64, 0, one, None), T.INVALID_ARG, "k = 0")
    status(L.tamoe_renorm_topk(one, 64, 9, one, None), T.UNSUPPORTED, "k = 9 exceeds")
    status(L.tamoe_renorm_topk(one, 64, 2, None, None), T.INVALID_ARG, "out is NULL")
    status(L.tamoe_renorm_topk_bwd(one, None, 64, 2, one, None), T.INVALID_ARG, "d_out is NULL")
    status(L.tamoe_dispatch_padded(one, one, None, 1, 64, 64, 8, 4, 2, 0, one, one, one, one, big, None),
           T.INVALID_ARG, "C = 0")
    status(L.tamoe_dispatch_padded(one, one, None, 1, 64, 64, 8, 4, 2, 1 << 29, one, one, one, one, big, None),
           T.INVALID_ARG, "N*C")
    status(L.tamoe_dispatch_padded(one, one, None, 1, 64, 64, 8, 4, 2, 16, None, one, one, one, big, None),
           T.INVALID_ARG, "send is NULL")
    status(L.tamoe_dispatch_padded(one, one, None, 1, 64, 64, 8, 4, 2, 16, one, one, one, one, 0, None),
           T.WORKSPACE_TOO_SMALL, "needed")


def test_workspace_size_is_monotone_and_covers_the_configs(T):
    prev = 0
    for S in (0, 1, 100, 4096, 65536):
        b = T.tamoe_workspace_bytes(S, 1024, 64, 64, 2, T.BF16)
        assert b >= prev and b % 256 == 0 and b > 0
        prev = b
    wl = W.WORKLOADS["large"]
    assert T.tamoe_workspace_bytes(wl.S, wl.d, wl.N, wl.P, wl.k, wl.dtype) < 64 << 20


def test_binding_has_no_cpu_fallback(T, monkeypatch):
    """A missing library must raise, never route anywhere else."""
    import paper_2302_09915_amd as pkg

    monkeypatch.setattr(pkg, "_lib", None)
    monkeypatch.setattr(pkg, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libtamoe.so"))
    with pytest.raises(ImportError):
        pkg.lib()
    src = open(os.path.join(ROOT, "paper_2302_09915_amd", "__init__.py")).read()
    assert "import oracle" not in src and "from oracle" not in src


def test_bind_notes_one_call_and_restores_the_library(T):
    import torch

    """bind() runs a binding function against a stand-in that only notes the call; whatever happens
    inside, the real library is back afterwards."""
    with pytest.raises(T.TamoeError):
        T.bind(lambda: None)                                   # no entry point called
    with pytest.raises(T.TamoeError):
        T.bind(T.tamoe_combine, None, 0, torch.zeros((4, 2), dtype=torch.int32), None, torch.zeros((4, 8)))
    assert T.lib().tamoe_version() == T.tamoe_version() > 0    # not the stand-in
    call = T.bind(T.tamoe_version)                              # a call whose result is not a status of 0
    with pytest.raises(T.TamoeError):
        call()
