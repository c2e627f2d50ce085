"""Parity of the variants of the path against the oracle: renormalised combine weights (forward and
transpose), the fixed-size zero-padded send layout, and the combine on that layout."""
import numpy as np
import pytest

import tamoe_workloads as W
from test_gpu_parity import check_combine, to_dev, to_host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    import paper_2302_09915_amd as T

    T.lib()
    return T


# ---- renormalised weights ----------------------------------------------------------------

@pytest.mark.parametrize("S,N,k", [(4096, 16, 2), (1000, 64, 1), (777, 32, 5), (16384, 128, 8), (1, 4, 3)])
def test_renorm_topk_matches_oracle(T, oracle, S, N, k):
    lg = W.random_logits(S + k, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    _, wgt = oracle.topk(lg, G, k)
    w32 = wgt.astype(np.float32)
    ref = oracle.renorm_topk(w32.astype(np.float64))
    wd = torch.from_numpy(w32).cuda()
    out = torch.empty_like(wd)
    T.tamoe_renorm_topk(wd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    # k-1 fp32 additions and one division: (k + 1) roundings of 2^-24 each at most
    np.testing.assert_allclose(got, ref, rtol=(k + 1) * 2.0 ** -24, atol=0)
    # in place
    T.tamoe_renorm_topk(wd, wd)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(wd.cpu().numpy(), got)


@pytest.mark.parametrize("S,k", [(4096, 2), (513, 1), (3000, 4), (100, 8)])
def test_renorm_topk_bwd_matches_oracle(T, oracle, S, k):
    rng = np.random.default_rng(S + k)
    w32 = rng.uniform(0.02, 1.0, size=(S, k)).astype(np.float32)
    g32 = rng.standard_normal((S, k)).astype(np.float32)
    ref = oracle.renorm_topk_bwd(w32.astype(np.float64), g32.astype(np.float64))
    wd, gd = torch.from_numpy(w32).cuda(), torch.from_numpy(g32).cuda()
    out = torch.empty_like(wd)
    T.tamoe_renorm_topk_bwd(wd, gd, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # the two terms g/s and (g.w)/s^2 cancel: the error is relative to their magnitudes, not to the result
    s = w32.astype(np.float64).sum(axis=1, keepdims=True)
    mag = np.abs(g32) / s + (np.abs(g32) * w32).sum(axis=1, keepdims=True) / s ** 2
    # roundings: k in the dot product, k in s, one in 1/s, two in dot/s^2, one in the final fma
    assert (np.abs(got - ref) <= (3 * k + 4) * 2.0 ** -24 * mag).all()
    if k == 1:
        assert (np.abs(got) <= 4 * 2.0 ** -24 * mag).all()      # one weight, always 1: no gradient


# ---- fixed-size padded layout -----------------------------------------------------------------

def _padded_case(T, oracle, S, d, N, P, k, C, dtype, cap, seed, skew=0.0):
    idx = W.random_routing(seed, S, N, k, skew=skew)
    rng = np.random.default_rng(seed)
    x_np = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    x = to_dev(x_np, dtype)
    ws = T.workspace(S, d, N, P, k, dtype)
    send = to_dev(W.to_storage(np.full((N * C, d), 7.0, dtype=np.float32), dtype), dtype)   # dirty buffer
    slot = torch.empty((S, k), dtype=torch.int32, device="cuda")
    kept = torch.empty((N,), dtype=torch.int32, device="cuda")
    cap_d = None if cap is None else torch.from_numpy(cap).cuda()
    T.tamoe_dispatch_padded(x, torch.from_numpy(idx).cuda(), cap_d, N, P, C, send, slot, kept, ws)
    torch.cuda.synchronize()
    ref_slot, ref_kept = oracle.slots_padded(idx, cap, N, C)
    np.testing.assert_array_equal(slot.cpu().numpy(), ref_slot)
    np.testing.assert_array_equal(kept.cpu().numpy(), ref_kept)
    ref_send = oracle.scatter(x_np, dtype, ref_slot, N * C)
    np.testing.assert_array_equal(to_host(send, dtype), ref_send)
    return x_np, idx, send, slot, ref_slot, ref_send


@pytest.mark.parametrize("S,d,N,P,k,C,dtype,with_cap", [
    (4096, 512, 16, 16, 2, 640, W.BF16, False),      # Small-shaped, C = its uniform capacity
    (3000, 264, 24, 8, 3, 100, W.BF16, True),        # ragged sizes, drops by cap and by C
    (512, 64, 8, 8, 1, 64, W.F32, False),            # Tiny-shaped
    (2048, 1024, 64, 64, 2, 77, W.BF16, True),
    (100, 8, 4, 2, 2, 1000, W.F32, True),            # C far above the load: mostly padding
    (1500, 776, 32, 8, 2, 90, W.F16, True),          # half precision
])
def test_dispatch_padded_matches_oracle(T, oracle, S, d, N, P, k, C, dtype, with_cap):
    cap = None
    if with_cap:
        cap = np.random.default_rng(S).integers(0, C + C // 2 + 1, size=N).astype(np.int32)
    x_np, idx, send, slot, ref_slot, ref_send = _padded_case(T, oracle, S, d, N, P, k, C, dtype, cap, seed=S + d,
                                                             skew=0.5)
    # combine works on the padded layout unchanged
    rng = np.random.default_rng(S)
    w32 = rng.uniform(0.05, 1.0, size=(S, k)).astype(np.float32)
    y = torch.empty((S, d), dtype=send.dtype, device="cuda")
    T.tamoe_combine(send, N * C, slot, torch.from_numpy(w32).cuda(), y)
    torch.cuda.synchronize()
    y_exact, y_ref = oracle.combine(ref_send, dtype, ref_slot, w32.astype(np.float64))
    rows = W.storage_to_f64(ref_send, dtype)
    mag = np.zeros((S, d))
    for j in range(k):
        live = ref_slot[:, j] >= 0
        mag[live] += np.abs(w32[live, j, None].astype(np.float64) * rows[ref_slot[live, j]])
    check_combine(to_host(y, dtype), y_exact, y_ref, mag, dtype, k)


def test_dispatch_padded_equals_packed_rows(T, oracle):
    """The padded buffer holds the packed buffer's rows, expert by expert, with zero rows between."""
    wl = W.WORKLOADS["gpt_moe"]
    S, d, N, P, k = 4096, wl.d, wl.N, wl.P, wl.k
    C = 160
    x_np, idx, send, slot, ref_slot, _ = _padded_case(T, oracle, S, d, N, P, k, C, wl.dtype, None, seed=5, skew=1.0)
    x = to_dev(x_np, wl.dtype)
    ws = T.workspace(S, d, N, P, k, wl.dtype)
    cap = torch.full((N,), C, dtype=torch.int32, device="cuda")
    dsp = T.dispatch(x, torch.from_numpy(idx).cuda(), cap, N, P, ws=ws)
    torch.cuda.synchronize()
    off = dsp["expert_offset"].cpu().numpy()
    packed = to_host(dsp["send"], wl.dtype)
    padded = to_host(send, wl.dtype)
    assert (off[1:] - off[:-1]).max() == C                      # the skew fills at least one expert
    for e in range(N):
        n = off[e + 1] - off[e]
        np.testing.assert_array_equal(padded[e * C:e * C + n], packed[off[e]:off[e + 1]])
        assert not padded[e * C + n:(e + 1) * C].any()


def test_dispatch_padded_empty_and_bad_arguments(T):
    ws = T.workspace(64, 64, 8, 4, 2, T.F32)
    x = torch.zeros((0, 64), device="cuda")
    idx = torch.zeros((0, 2), dtype=torch.int32, device="cuda")
    send = torch.ones((8 * 3, 64), device="cuda")
    slot = torch.empty((0, 2), dtype=torch.int32, device="cuda")
    kept = torch.full((8,), -1, dtype=torch.int32, device="cuda")
    T.tamoe_dispatch_padded(x, idx, None, 8, 4, 3, send, slot, kept, ws)
    torch.cuda.synchronize()
    assert not send.any().item() and not kept.any().item()       # no tokens: all padding
    x = torch.zeros((64, 64), device="cuda")
    idx = torch.zeros((64, 2), dtype=torch.int32, device="cuda")
    slot = torch.empty((64, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(T.TamoeError) as ei:
        T.tamoe_dispatch_padded(x, idx, None, 8, 4, 4, send, slot, kept, ws)    # send has 8*3 rows
    assert ei.value.status == T.INVALID_ARG
    L = T.lib()
    rc = L.tamoe_dispatch_padded(x.data_ptr(), idx.data_ptr(), None, T.F32, 64, 64, 8, 4, 2, 0, send.data_ptr(),
                                 slot.data_ptr(), kept.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert rc == T.INVALID_ARG and "C = 0" in T.tamoe_last_error()


def test_dispatch_padded_at_the_benchmarked_size(T, oracle):
    """Large: 65536 tokens of 8 KiB, 128 experts, top-2, C = the uniform capacity 1280; slots and every
    row of the 1.25 GiB buffer compared."""
    wl = W.WORKLOADS["large"]
    S, d, N, P, k, C = wl.S, wl.d, wl.N, wl.P, wl.k, 1280
    oracle.set_threads(oracle.max_threads())
    idx = W.random_routing(21, S, N, k, skew=0.3)
    rng = np.random.Generator(np.random.Philox(key=[4, 12]))
    x_np = rng.integers(0, 1 << 16, size=(S, d), dtype=np.uint16)
    x_np[x_np == 0] = 1                                                  # no all-zero rows: padding is recognisable
    x = torch.from_numpy(x_np.view(np.int16)).cuda().view(torch.bfloat16)
    ws = T.workspace(S, d, N, P, k, wl.dtype)
    send = torch.full((N * C, d), 3.0, dtype=torch.bfloat16, device="cuda")
    slot = torch.empty((S, k), dtype=torch.int32, device="cuda")
    kept = torch.empty((N,), dtype=torch.int32, device="cuda")
    T.tamoe_dispatch_padded(x, torch.from_numpy(idx).cuda(), None, N, P, C, send, slot, kept, ws)
    torch.cuda.synchronize()
    ref_slot, ref_kept = oracle.slots_padded(idx, None, N, C)
    np.testing.assert_array_equal(slot.cpu().numpy(), ref_slot)
    np.testing.assert_array_equal(kept.cpu().numpy(), ref_kept)
    assert ref_kept.max() == C and ref_kept.min() < C                    # some experts overflow, some have padding
    ref_send = oracle.scatter(x_np, wl.dtype, ref_slot, N * C)
    assert np.array_equal(to_host(send, wl.dtype), ref_send)
