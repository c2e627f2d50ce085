"""Parity of the backward entry points (through the C ABI) against the CPU oracle on an MI355X.

Tolerances (derived from the arithmetic):
  d_logits  = G * (u - sum u G) in fp32 with the hardware exp2; the subtraction cancels when the
            u[e] are close to each other, so the bound is relative to the magnitude before it:
            |d - ref| <= 1e-5 * G[t][e] * (|u[t][e]| + sum_e' |u[t][e']| G[t][e']);
  d_recv    one fp32 product rounded once to the storage type: within half an ulp of the storage
            type of the exact product (+ one fp32 rounding), bit-equal to the oracle's once-rounded
            value in all but <= 1e-3 of the elements (bf16);
  d_topk_w  fp32 dot product over d terms: |d - ref| <= 1e-5 * sum_q |dy*recv| (+ tiny absolute);
  d_x       like the combine with unit weights.
"""
import math

import numpy as np
import pytest

import tamoe_workloads as W
from test_gpu_parity import check_combine, flip_bound, to_dev, to_host, torch_dtype, ulp_of

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    import paper_2302_09915_amd as T

    T.lib()
    return T


def dlogits_bound(oracle, lg, idx, dw, pen, c, loss_scale, P):
    """1e-5 times the magnitude of G * (u - ubar) before the cancellation."""
    S, N = lg.shape
    G = oracle.softmax(lg.astype(np.float64))
    coef = loss_scale * (N * P * pen.astype(np.float64) if pen is not None else 1.0) * c / float(S) ** 2
    u = np.tile(np.abs(coef), (S, 1))
    for j in range(idx.shape[1]):
        np.add.at(u, (np.arange(S), idx[:, j]), np.abs(dw[:, j].astype(np.float64)))
    return 1e-5 * G * (u + (u * G).sum(axis=1, keepdims=True)) + 1e-35


def random_slots(rng, S, k, K, drop=0.2):
    """Every row 0..K-1 named by exactly one pair (K <= S*k); the other pairs are dropped (-1)."""
    flat = -np.ones(S * k, dtype=np.int32)
    pos = rng.choice(S * k, size=K, replace=False)
    flat[pos] = rng.permutation(K).astype(np.int32)
    return flat.reshape(S, k)


@pytest.mark.parametrize("S,N,P,k,use_penalty", [
    (1000, 16, 4, 2, True), (777, 64, 64, 2, True), (513, 128, 64, 4, True), (4000, 8, 8, 1, False),
    (100, 48, 16, 3, True), (1, 2, 1, 1, True), (2100, 128, 1, 8, False)])
def test_gate_bwd(T, oracle, S, N, P, k, use_penalty):
    rng = np.random.default_rng(S + N)
    lg = W.random_logits(S, S, N)
    G = oracle.softmax(lg.astype(np.float64))
    idx, _ = oracle.topk(lg.astype(np.float64), G, k)
    c = np.bincount(idx.ravel(), minlength=N).astype(np.int32)
    dw = rng.standard_normal((S, k)).astype(np.float32)
    pen = None
    if use_penalty:
        beta = rng.uniform(1.0, 9.0, size=(P, P))
        _, pen, _ = T.tamoe_topo_pattern(beta, None, P, N, P // 2, k, S, 1.0, 0)
    out = torch.empty((S, N), dtype=torch.float32, device="cuda")
    T.tamoe_gate_bwd(torch.from_numpy(lg).cuda(), torch.from_numpy(idx).cuda(), torch.from_numpy(dw).cuda(),
                     None if pen is None else torch.from_numpy(pen).cuda(), torch.from_numpy(c).cuda(), 1.0, P, out)
    torch.cuda.synchronize()
    ref = oracle.gate_bwd(lg.astype(np.float64), idx, dw.astype(np.float64),
                          None if pen is None else pen.astype(np.float64), c, 1.0, P)
    got = out.cpu().numpy().astype(np.float64)
    assert (np.abs(got - ref) <= dlogits_bound(oracle, lg, idx, dw, pen, c, 1.0, P)).all()
    # the loss term alone (zero weight gradients) at a scale of 1000: same relative accuracy
    zero = torch.zeros((S, k), dtype=torch.float32, device="cuda")
    T.tamoe_gate_bwd(torch.from_numpy(lg).cuda(), torch.from_numpy(idx).cuda(), zero,
                     None if pen is None else torch.from_numpy(pen).cuda(), torch.from_numpy(c).cuda(), 1000.0, P, out)
    torch.cuda.synchronize()
    ref0 = oracle.gate_bwd(lg.astype(np.float64), idx, np.zeros((S, k)),
                           None if pen is None else pen.astype(np.float64), c, 1000.0, P)
    got0 = out.cpu().numpy().astype(np.float64)
    assert (np.abs(got0 - ref0) <= dlogits_bound(oracle, lg, idx, np.zeros((S, k)), pen, c, 1000.0, P)).all()


@pytest.mark.parametrize("dtype,S,d,k,frac", [
    (W.BF16, 3000, 136, 2, 0.8), (W.BF16, 700, 4096, 2, 1.0), (W.BF16, 5000, 512, 1, 0.5),
    (W.F32, 900, 36, 3, 0.7), (W.BF16, 333, 1032, 5, 0.6), (W.F32, 1, 4, 1, 1.0),
    # rows of 2^n KiB with k <= 2 take the one-chunk-per-thread kernel: 2, 8 and 16 KiB rows, a last
    # workgroup that is partly empty, both storage types
    (W.BF16, 1001, 1024, 2, 0.7), (W.F32, 513, 2048, 2, 0.9), (W.BF16, 131, 8192, 1, 0.8), (W.F32, 67, 256, 2, 0.5),
    # half precision: both kernels
    (W.F16, 900, 1024, 2, 0.8), (W.F16, 333, 1032, 3, 0.6), (W.F16, 500, 4096, 1, 1.0)])
def test_combine_bwd_and_dispatch_bwd(T, oracle, dtype, S, d, k, frac):
    oracle.set_threads(oracle.max_threads())
    rng = np.random.default_rng(S + d)
    K = max(1, int(S * k * frac))
    slot = random_slots(rng, S, k, K)
    recv = W.to_storage(rng.standard_normal((K, d)).astype(np.float32), dtype)
    dy = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    wgt = rng.uniform(0.05, 1.0, size=(S, k)).astype(np.float32)
    dev = "cuda"
    d_recv = torch.zeros((K, d), dtype=torch_dtype(dtype), device=dev)
    d_w = torch.full((S, k), 7.0, dtype=torch.float32, device=dev)
    slot_d, wgt_d = torch.from_numpy(slot).cuda(), torch.from_numpy(wgt).cuda()
    T.tamoe_combine_bwd(to_dev(dy, dtype), to_dev(recv, dtype), K, slot_d, wgt_d, d_recv, d_w)
    torch.cuda.synchronize()
    ex, rounded, dw_ref = oracle.combine_bwd(dy, recv, dtype, slot, wgt.astype(np.float64))
    got = to_host(d_recv, dtype)
    gv = W.storage_to_f64(got, dtype)
    # exact product -> fp32 -> storage: half an ulp of the storage type plus one fp32 rounding
    assert (np.abs(gv - ex) <= 0.5 * ulp_of(ex, dtype) + 2.0 ** -23 * np.abs(ex) + 2.0 ** -149).all()
    if dtype != W.F32:
        assert (got != rounded).mean() <= flip_bound(dtype, 1)
    dyv, rv = np.abs(W.storage_to_f64(dy, dtype)), np.abs(W.storage_to_f64(recv, dtype))
    mag = np.zeros((S, k))
    for j in range(k):
        ok = slot[:, j] >= 0
        mag[ok, j] = (dyv[ok] * rv[slot[ok, j]]).sum(axis=1)
    gw = d_w.cpu().numpy().astype(np.float64)
    assert (np.abs(gw - dw_ref) <= 1e-5 * mag + 1e-30).all()
    assert (gw[slot < 0] == 0).all()

    # transpose of the scatter on the same slots
    d_send = W.to_storage(rng.standard_normal((K, d)).astype(np.float32), dtype)
    d_x = torch.empty((S, d), dtype=d_recv.dtype, device=dev)
    T.tamoe_dispatch_bwd(to_dev(d_send, dtype), K, slot_d, d_x)
    torch.cuda.synchronize()
    dx_exact, dx_ref = oracle.dispatch_bwd(d_send, dtype, slot)
    sv = np.abs(W.storage_to_f64(d_send, dtype))
    mag2 = np.zeros((S, d))
    for j in range(k):
        ok = slot[:, j] >= 0
        mag2[ok] += sv[slot[ok, j]]
    check_combine(to_host(d_x, dtype), dx_exact, dx_ref, mag2, dtype, k)


def test_backward_chain_on_the_small_config(T, oracle):
    """Forward on the GPU, then the three backward calls; every piece against the oracle fed the
    GPU's own forward results."""
    wl = W.WORKLOADS["small"]
    oracle.set_threads(oracle.max_threads())
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    _, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    cap = (cap // 4).astype(np.int32)                      # force drops, some tokens lose both choices
    x, w = to_dev(inp["x"], wl.dtype), to_dev(inp["w"], wl.dtype)
    g = T.gate(x, w, wl.P, wl.k)
    dsp = T.dispatch(x, g["topk_idx"], torch.from_numpy(cap).cuda(), wl.N, wl.P)
    torch.cuda.synchronize()
    K = int(dsp["expert_offset"][-1].item())
    assert K < wl.S * wl.k
    rng = np.random.default_rng(0)
    dy = W.to_storage(rng.standard_normal((wl.S, wl.d)).astype(np.float32), wl.dtype)
    dy_d = to_dev(dy, wl.dtype)
    recv = dsp["send"][:K].contiguous()
    d_recv = torch.empty_like(recv)
    d_w = torch.empty((wl.S, wl.k), dtype=torch.float32, device="cuda")
    T.tamoe_combine_bwd(dy_d, recv, K, dsp["slot"], g["topk_w"], d_recv, d_w)
    d_logits = torch.empty((wl.S, wl.N), dtype=torch.float32, device="cuda")
    T.tamoe_gate_bwd(g["logits"], g["topk_idx"], d_w, torch.from_numpy(pen).cuda(), g["c_expert"], 1.0, wl.P, d_logits)
    d_x = torch.empty_like(x)
    T.tamoe_dispatch_bwd(d_recv, K, dsp["slot"], d_x)      # identity expert: d_send = d_recv
    torch.cuda.synchronize()

    slot = dsp["slot"].cpu().numpy()
    wg = g["topk_w"].cpu().numpy().astype(np.float64)
    recv_h = to_host(recv, wl.dtype)
    ex, rounded, dw_ref = oracle.combine_bwd(dy, recv_h, wl.dtype, slot, wg)
    assert (to_host(d_recv, wl.dtype) != rounded).mean() <= 1e-3
    gw = d_w.cpu().numpy()
    ref_dl = oracle.gate_bwd(g["logits"].cpu().numpy().astype(np.float64), g["topk_idx"].cpu().numpy(),
                             gw.astype(np.float64), pen.astype(np.float64), g["c_expert"].cpu().numpy(), 1.0, wl.P)
    got_dl = d_logits.cpu().numpy().astype(np.float64)
    bound = dlogits_bound(oracle, g["logits"].cpu().numpy(), g["topk_idx"].cpu().numpy(), gw, pen,
                          g["c_expert"].cpu().numpy(), 1.0, wl.P)
    assert (np.abs(got_dl - ref_dl) <= bound).all()
    dx_exact, dx_ref = oracle.dispatch_bwd(to_host(d_recv, wl.dtype), wl.dtype, slot)
    assert (to_host(d_x, wl.dtype) != dx_ref).mean() <= 1e-3
    dead = (slot < 0).all(axis=1)
    assert dead.any() and (W.storage_to_f64(to_host(d_x, wl.dtype), wl.dtype)[dead] == 0).all()


def test_backward_rejects_bad_arguments(T):
    z = torch.zeros((4, 8), dtype=torch.float32, device="cuda")
    i = torch.zeros((4, 2), dtype=torch.int32, device="cuda")
    c = torch.zeros((8,), dtype=torch.int32, device="cuda")
    with pytest.raises(T.TamoeError) as ei:
        T.tamoe_gate_bwd(z, i, z[:, :2].contiguous(), None, c, 1.0, 3, z.clone())       # N % P != 0
    assert ei.value.status == T.INVALID_ARG
    with pytest.raises(T.TamoeError):
        T.tamoe_dispatch_bwd(z, 4, i, torch.zeros((4, 6), dtype=torch.float32, device="cuda"))  # 24-byte rows
