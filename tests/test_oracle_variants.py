"""Pins for the oracle's variants of the path: the softmax-type Norm of the penalty (Section 4.3),
combine weights renormalised over the k selected experts, and the fixed-size zero-padded send
layout that the paper's variable chunk sizes replace (Section 4.3)."""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import tamoe_workloads as W


# ---- softmax Norm -------------------------------------------------------------

def test_softmax_norm_two_experts_is_the_logistic_function(oracle):
    # N = 2: r = (2a/(a+b), 2b/(a+b)) with a = 1/c0, b = 1/c1, p0 = 1 / (1 + exp(tau (r1 - r0)))
    c_hat = np.array([3.0, 12.0])
    a, b = 1 / 3.0, 1 / 12.0
    for tau in (0.5, 1.0, 3.0):
        p = oracle.penalty_softmax(c_hat, tau)
        expect0 = 1.0 / (1.0 + np.exp(tau * (2 * b - 2 * a) / (a + b)))
        assert p[0] == pytest.approx(expect0, rel=1e-14)
        assert p[1] == pytest.approx(1.0 - expect0, rel=1e-13)


def test_softmax_norm_properties(oracle):
    rng = np.random.default_rng(3)
    c_hat = rng.uniform(1.0, 50.0, size=24)
    for tau in (0.0, 0.7, 2.5, 40.0):
        p = oracle.penalty_softmax(c_hat, tau)
        assert p.sum() == pytest.approx(1.0, rel=1e-14)
        assert np.all(p > 0) or tau == 40.0
        # the smaller the target volume (the slower the link), the larger the penalty
        order = np.argsort(c_hat)
        assert np.all(np.diff(p[order]) <= 1e-18)
        # scale-free: the pattern's unit (tokens) does not matter
        np.testing.assert_allclose(oracle.penalty_softmax(c_hat * 123.0, tau), p, rtol=1e-12)
    np.testing.assert_allclose(oracle.penalty_softmax(c_hat, 0.0), np.full(24, 1 / 24), rtol=1e-15)


def test_softmax_norm_is_library_softmax_of_the_scaled_l1_norm(oracle):
    # r = N * (L1-normalised inverse pattern): the oracle's own L1 Norm is pinned elsewhere
    rng = np.random.default_rng(4)
    c_hat = rng.uniform(0.5, 9.0, size=16)
    inv = 1.0 / c_hat
    r = inv / inv.sum() * 16
    for tau in (0.3, 1.0, 5.0):
        np.testing.assert_allclose(oracle.penalty_softmax(c_hat, tau), scipy_softmax(tau * r), rtol=1e-12)


def test_softmax_norm_enlarges_the_slow_link_penalty_beyond_a_threshold(oracle):
    # two-tier pattern, ratio rho: L1 gives p_slow/p_fast = rho; softmax gives exp(tau (r_slow - r_fast)),
    # which exceeds rho exactly when tau > ln(rho) / (r_slow - r_fast)
    beta, level = W.two_tier_topology(2, 4, 4.0)
    beta_hat = oracle.smooth_beta(beta, level)
    c_hat = oracle.target_pattern(beta_hat, 8, 0, 1, 512)
    inv = 1.0 / c_hat
    r = inv / inv.mean()
    tau_star = np.log(4.0) / (r.max() - r.min())
    lo = oracle.penalty_softmax(c_hat, 0.9 * tau_star)
    hi = oracle.penalty_softmax(c_hat, 1.1 * tau_star)
    assert lo.max() / lo.min() < 4.0 < hi.max() / hi.min()
    assert hi.max() / hi.min() == pytest.approx(4.0 ** 1.1, rel=1e-12)


def test_softmax_norm_large_tau_does_not_overflow(oracle):
    p = oracle.penalty_softmax(np.array([1.0, 1.0, 1e-3]), 1e4)
    assert np.isfinite(p).all() and p[2] == pytest.approx(1.0)


# ---- renormalised combine weights ------------------------------------------------

def test_renorm_rows_sum_to_one_and_keep_ratios(oracle):
    rng = np.random.default_rng(5)
    w = rng.uniform(0.01, 1.0, size=(50, 3))
    out = oracle.renorm_topk(w)
    np.testing.assert_allclose(out.sum(axis=1), 1.0, rtol=1e-15)
    np.testing.assert_allclose(out[:, 0] / out[:, 2], w[:, 0] / w[:, 2], rtol=1e-14)
    np.testing.assert_array_equal(oracle.renorm_topk(w[:, :1]), np.ones((50, 1)))


def test_renorm_of_gate_weights_is_softmax_over_the_selected_scores(oracle):
    lg = W.random_logits(6, 64, 16).astype(np.float64)
    G = oracle.softmax(lg)
    idx, wgt = oracle.topk(lg, G, 4)
    sel = np.take_along_axis(lg, idx.astype(np.int64), axis=1)
    np.testing.assert_allclose(oracle.renorm_topk(wgt), scipy_softmax(sel, axis=1), rtol=1e-12)


def test_renorm_bwd_finite_differences_and_null_direction(oracle):
    rng = np.random.default_rng(7)
    w = rng.uniform(0.05, 1.0, size=(6, 3))
    g = rng.standard_normal((6, 3))
    dw = oracle.renorm_topk_bwd(w, g)
    h = 1e-6
    for t in range(6):
        for i in range(3):
            wp, wm = w.copy(), w.copy()
            wp[t, i] += h
            wm[t, i] -= h
            fd = ((oracle.renorm_topk(wp) - oracle.renorm_topk(wm)) * g).sum() / (2 * h)
            assert dw[t, i] == pytest.approx(fd, rel=1e-6, abs=1e-8)
    # scaling a token's weights does not change the output: the gradient is orthogonal to w
    np.testing.assert_allclose((dw * w).sum(axis=1), 0.0, atol=1e-14)
    # a gradient that is constant over j cannot move weights that sum to one
    np.testing.assert_allclose(oracle.renorm_topk_bwd(w, np.ones_like(w)), 0.0, atol=1e-14)


# ---- fixed-size padded layout -----------------------------------------------------

def _brute_padded(idx, cap, N, C):
    S, k = idx.shape
    slot = -np.ones((S, k), dtype=np.int64)
    seen = [0] * N
    for j in range(k):
        for t in range(S):
            e = int(idx[t, j])
            lim = C if cap is None else min(C, int(cap[e]))
            if seen[e] < lim:
                slot[t, j] = e * C + seen[e]
            seen[e] += 1
    return slot


@pytest.mark.parametrize("S,N,k,C,with_cap", [(40, 4, 2, 8, False), (64, 8, 1, 5, True), (33, 3, 3, 40, True),
                                              (1, 2, 1, 1, False)])
def test_padded_slots_brute_force(oracle, S, N, k, C, with_cap):
    idx = W.random_routing(S + N, S, N, k)
    cap = None
    if with_cap:
        cap = np.random.default_rng(S).integers(0, C + 4, size=N).astype(np.int32)
    slot, kept = oracle.slots_padded(idx, cap, N, C)
    np.testing.assert_array_equal(slot, _brute_padded(idx, cap, N, C))
    live = slot[slot >= 0]
    assert len(np.unique(live)) == len(live)
    c = np.bincount(idx.ravel(), minlength=N)
    lim = np.full(N, C) if cap is None else np.minimum(cap, C)
    np.testing.assert_array_equal(kept, np.minimum(c, lim))
    np.testing.assert_array_equal(np.bincount(live // C, minlength=N), kept)


def test_padded_buffer_is_the_packed_buffer_with_zero_rows_between(oracle):
    S, N, k, d, P = 96, 8, 2, 8, 4
    idx = W.random_routing(11, S, N, k)
    cap = np.array([30, 5, 17, 0, 40, 12, 24, 9], dtype=np.int32)
    C = 24
    x = np.random.default_rng(12).standard_normal((S, d)).astype(np.float32)
    x[np.abs(x) < 1e-3] = 0.5                                  # no zero entries: padding is recognisable
    slot_p, kept_p = oracle.slots_padded(idx, cap, N, C)
    pad = oracle.scatter(x, W.F32, slot_p, N * C)
    slot, kept, off, _, K = oracle.slots(idx, np.minimum(cap, C).astype(np.int32), P)
    packed = oracle.scatter(x, W.F32, slot, K)
    np.testing.assert_array_equal(kept_p, kept)
    for e in range(N):
        np.testing.assert_array_equal(pad[e * C:e * C + kept[e]], packed[off[e]:off[e + 1]])
        assert not pad[e * C + kept[e]:(e + 1) * C].any()
    # same combine result through either layout (identity experts)
    w = np.random.default_rng(13).uniform(0.1, 1.0, size=(S, k))
    y_pad, _ = oracle.combine(pad, W.F32, slot_p, w, want_rounded=False)
    y_packed, _ = oracle.combine(packed, W.F32, slot, w, want_rounded=False)
    np.testing.assert_array_equal(y_pad, y_packed)
