"""Pins for the oracle's half-precision storage type (the FP16 of the paper's GPT model table): the
decoding of all 65536 bit patterns and the single rounding from double against numpy's float16, the
ties and range ends spelled out, and the path's row movers and weighted sums on half-precision rows."""
import numpy as np
import pytest

import tamoe_workloads as W


def test_every_half_bit_pattern_decodes_like_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_value(int(b)) for b in bits])
    both_nan = np.isnan(ref) & np.isnan(got)
    assert ((got == ref) | both_nan).all()
    assert (np.signbit(got) == np.signbit(ref))[~both_nan].all()          # -0.0 keeps its sign


def test_rounding_from_double_matches_numpy_float16(oracle):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 6, size=4000),   # normals, subnormals, overflow
        rng.uniform(-7e-5, 7e-5, size=2000),                                   # around the subnormal boundary 2^-14
        rng.uniform(60000, 70000, size=500) * rng.choice([-1, 1], size=500),  # around the largest finite value 65504
        [0.0, -0.0, 2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -14, 65504.0, 65519.99, 65520.0, -65520.0, 1e30],
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)                         # numpy rounds double -> half in one step
    got = np.array([oracle.round_to_f16(float(v)) for v in vals], dtype=np.uint16)
    np.testing.assert_array_equal(got, ref)


def test_half_ties_go_to_even_and_double_rounding_is_avoided(oracle):
    assert oracle.round_to_f16(1.0 + 2.0 ** -11) == 0x3C00                    # halfway 1 .. 1+2^-10: even is 1
    assert oracle.round_to_f16(1.0 + 3 * 2.0 ** -11) == 0x3C02                # halfway: even is 1+2*2^-10
    # just above the tie: a detour through float32 would first round down to the tie, then to even
    assert oracle.round_to_f16(1.0 + 2.0 ** -11 + 2.0 ** -40) == 0x3C01
    assert oracle.round_to_f16(-(1.0 + 2.0 ** -11 + 2.0 ** -40)) == 0xBC01
    assert oracle.round_to_f16(2.0 ** -25) == 0x0000                          # half of the smallest subnormal: tie to even (0)
    assert oracle.round_to_f16(2.0 ** -25 * 1.0000001) == 0x0001
    assert oracle.round_to_f16(float("inf")) == 0x7C00 and oracle.round_to_f16(-1e9) == 0xFC00
    assert oracle.half_value(0x7BFF) == 65504.0 and oracle.half_value(0x0001) == 2.0 ** -24


def test_workload_half_storage_round_trips(oracle):
    a = np.random.default_rng(1).standard_normal(5000).astype(np.float32) * 50
    bits = W.to_storage(a, W.F16)
    assert bits.dtype == np.uint16
    back = W.storage_to_f64(bits, W.F16)
    np.testing.assert_array_equal(back, a.astype(np.float16).astype(np.float64))
    np.testing.assert_array_equal(np.array([oracle.half_value(int(b)) for b in bits[:300]]), back[:300])


def test_path_on_half_rows(oracle):
    """Scores, scatter and combine on half-precision storage: the scores against numpy's float64 product of
    the decoded values, the scatter as a bit copy, the combine against the same sum rounded by numpy."""
    rng = np.random.default_rng(2)
    S, d, N, k, P = 70, 24, 6, 2, 3
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), W.F16)
    w = W.to_storage((rng.standard_normal((N, d)) / 5).astype(np.float32), W.F16)
    lg = oracle.logits(x, w, W.F16)
    np.testing.assert_allclose(lg, W.storage_to_f64(x, W.F16) @ W.storage_to_f64(w, W.F16).T, rtol=1e-13, atol=1e-14)
    r = oracle.route_from_logits(lg, k, P, np.full(N, 1 / N), np.full(N, 20, dtype=np.int32))
    send = oracle.scatter(x, W.F16, r["slot"], r["K"])
    for t in range(S):
        for j in range(k):
            if r["slot"][t, j] >= 0:
                np.testing.assert_array_equal(send[r["slot"][t, j]], x[t])
    y_exact, y = oracle.combine(send, W.F16, r["slot"], r["topk_w"])
    xv = W.storage_to_f64(x, W.F16)
    ref = np.zeros((S, d))
    for j in range(k):
        live = r["slot"][:, j] >= 0
        ref[live] += r["topk_w"][live, j, None] * xv[live]
    np.testing.assert_allclose(y_exact, ref, rtol=1e-14, atol=1e-300)
    np.testing.assert_array_equal(y, y_exact.astype(np.float16).view(np.uint16))
    # transposes on half rows: adjoint identity with exact (unrounded) outputs
    dy = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), W.F16)
    d_recv, _, d_w = oracle.combine_bwd(dy, send, W.F16, r["slot"], r["topk_w"], want_rounded=False)
    lhs = (W.storage_to_f64(dy, W.F16) * y_exact).sum()
    assert lhs == pytest.approx((d_w * r["topk_w"]).sum(), rel=1e-12)
    assert lhs == pytest.approx((d_recv * W.storage_to_f64(send, W.F16)).sum(), rel=1e-12)
