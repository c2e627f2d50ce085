"""Pins for the oracle's backward functions: finite differences of the oracle's own forward
functions (which are pinned elsewhere) and adjoint identities.  No formula is retyped."""
import numpy as np
import pytest

import tamoe_workloads as W


def _setup(oracle, S=23, P=4, E=2, k=2, capv=9, seed=0):
    N = P * E
    lg = W.random_logits(seed, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    idx, wgt = oracle.topk(lg, G, k)
    c_e, _, m = oracle.counts(idx, G, P)
    cap = np.full(N, capv, dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    beta, _ = W.two_tier_topology(2, P // 2, 6.0) if P > 1 else (np.ones((1, 1)), None)
    p = oracle.penalty(oracle.target_pattern(beta, N, 1 % P, k, S))
    return dict(S=S, N=N, P=P, k=k, lg=lg, idx=idx, wgt=wgt, c=c_e, slot=slot, K=K, p=p)


def _l_topo_of(oracle, lg, q):
    G = oracle.softmax(lg)
    m = G.mean(axis=0)
    return oracle.l_topo(q["p"], m, q["c"], q["P"], q["S"])


def test_loss_gradient_matches_finite_differences(oracle):
    q = _setup(oracle)
    zero = np.zeros((q["S"], q["k"]))
    g = oracle.gate_bwd(q["lg"], q["idx"], zero, q["p"], q["c"], 1.0, q["P"])
    rng = np.random.default_rng(1)
    h = 1e-6
    for _ in range(25):
        t, e = rng.integers(q["S"]), rng.integers(q["N"])
        lp, lm = q["lg"].copy(), q["lg"].copy()
        lp[t, e] += h
        lm[t, e] -= h
        fd = (_l_topo_of(oracle, lp, q) - _l_topo_of(oracle, lm, q)) / (2 * h)
        assert g[t, e] == pytest.approx(fd, rel=1e-6, abs=1e-11)
    # rows of a softmax gradient sum to zero; the scale is linear
    np.testing.assert_allclose(g.sum(axis=1), 0.0, atol=1e-15)
    g3 = oracle.gate_bwd(q["lg"], q["idx"], zero, q["p"], q["c"], 3.0, q["P"])
    np.testing.assert_allclose(g3, 3.0 * g, rtol=1e-13)


def test_l_aux_gradient_when_no_penalty_is_given(oracle):
    q = _setup(oracle, seed=3)
    zero = np.zeros((q["S"], q["k"]))
    g = oracle.gate_bwd(q["lg"], q["idx"], zero, None, q["c"], 1.0, q["P"])
    h = 1e-6
    for t, e in [(0, 0), (5, 3), (22, 7)]:
        lp, lm = q["lg"].copy(), q["lg"].copy()
        lp[t, e] += h
        lm[t, e] -= h
        f = lambda l: oracle.l_aux(oracle.softmax(l).mean(axis=0), q["c"], q["S"])
        assert g[t, e] == pytest.approx((f(lp) - f(lm)) / (2 * h), rel=1e-6, abs=1e-11)


def test_weight_gradient_path_matches_finite_differences(oracle):
    """L = sum dwgt * G[t, idx[t,j]] (what the combine hands back) for fixed routing."""
    q = _setup(oracle, seed=5)
    rng = np.random.default_rng(2)
    dw = rng.standard_normal((q["S"], q["k"]))
    g = oracle.gate_bwd(q["lg"], q["idx"], dw, q["p"], q["c"], 0.0, q["P"])

    def f(l):
        G = oracle.softmax(l)
        return float((dw * np.take_along_axis(G, q["idx"].astype(np.int64), axis=1)).sum())

    h = 1e-6
    for _ in range(25):
        t, e = rng.integers(q["S"]), rng.integers(q["N"])
        lp, lm = q["lg"].copy(), q["lg"].copy()
        lp[t, e] += h
        lm[t, e] -= h
        assert g[t, e] == pytest.approx((f(lp) - f(lm)) / (2 * h), rel=1e-6, abs=1e-10)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_dispatch_backward_is_the_transpose_of_the_scatter(oracle, dtype):
    """<dsend, scatter(x)> == <dispatch_bwd(dsend), x> for any x, dsend."""
    q = _setup(oracle, S=40, capv=7, seed=7)
    d = 8
    rng = np.random.default_rng(3)
    x = W.to_storage(rng.standard_normal((q["S"], d)).astype(np.float32), dtype)
    dsend = W.to_storage(rng.standard_normal((q["K"], d)).astype(np.float32), dtype)
    send = oracle.scatter(x, dtype, q["slot"], q["K"])
    dx_exact, dx = oracle.dispatch_bwd(dsend, dtype, q["slot"])
    lhs = (W.storage_to_f64(dsend, dtype) * W.storage_to_f64(send, dtype)).sum()
    rhs = (dx_exact * W.storage_to_f64(x, dtype)).sum()
    assert lhs == pytest.approx(rhs, rel=1e-13)
    dead = (q["slot"] < 0).all(axis=1)
    assert dead.any() and (dx_exact[dead] == 0).all()
    if dtype == W.F32:
        np.testing.assert_array_equal(dx, dx_exact.astype(np.float32))


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_combine_backward_adjoint_and_weight_gradient(oracle, dtype):
    q = _setup(oracle, S=40, capv=7, seed=9)
    d = 8
    rng = np.random.default_rng(4)
    recv = W.to_storage(rng.standard_normal((q["K"], d)).astype(np.float32), dtype)
    dy = W.to_storage(rng.standard_normal((q["S"], d)).astype(np.float32), dtype)
    y_exact, _ = oracle.combine(recv, dtype, q["slot"], q["wgt"])
    drecv_exact, drecv, dwgt = oracle.combine_bwd(dy, recv, dtype, q["slot"], q["wgt"])
    dyv, rv = W.storage_to_f64(dy, dtype), W.storage_to_f64(recv, dtype)
    # linear in recv: <dy, y> == <drecv, recv>
    assert (dyv * y_exact).sum() == pytest.approx((drecv_exact * rv).sum(), rel=1e-13)
    # and in the weights: <dy, y> == <dwgt, wgt> (dropped pairs contribute nothing)
    assert (dyv * y_exact).sum() == pytest.approx((dwgt * q["wgt"]).sum(), rel=1e-13)
    assert (dwgt[q["slot"] < 0] == 0).all()
    # finite difference in one weight
    h = 1e-6
    for t, j in [(0, 0), (7, 1), (39, 0)]:
        wp, wm = q["wgt"].copy(), q["wgt"].copy()
        wp[t, j] += h
        wm[t, j] -= h
        f = lambda w: (dyv * oracle.combine(recv, dtype, q["slot"], w)[0]).sum()
        assert dwgt[t, j] == pytest.approx((f(wp) - f(wm)) / (2 * h), rel=1e-6, abs=1e-9)
    # every send-buffer row is named by exactly one kept pair, so no row of drecv stays zero by accident
    named = np.zeros(q["K"], dtype=bool)
    named[q["slot"][q["slot"] >= 0]] = True
    assert named.all()
    if dtype == W.F32:
        np.testing.assert_array_equal(drecv, drecv_exact.astype(np.float32))


def test_whole_backward_chain_matches_finite_differences(oracle):
    """L(logits) = <dy, combine(recv; w(logits))> + l_topo(logits), routing fixed."""
    q = _setup(oracle, S=17, capv=6, seed=11)
    d = 6
    rng = np.random.default_rng(5)
    recv = rng.standard_normal((q["K"], d)).astype(np.float32)
    dy = rng.standard_normal((q["S"], d)).astype(np.float32)
    _, _, dwgt = oracle.combine_bwd(dy, recv, W.F32, q["slot"], q["wgt"])
    g = oracle.gate_bwd(q["lg"], q["idx"], dwgt, q["p"], q["c"], 1.0, q["P"])

    def L(l):
        G = oracle.softmax(l)
        w = np.take_along_axis(G, q["idx"].astype(np.int64), axis=1)
        y, _ = oracle.combine(recv, W.F32, q["slot"], w)
        return float((dy.astype(np.float64) * y).sum()) + oracle.l_topo(q["p"], G.mean(axis=0), q["c"], q["P"], q["S"])

    h = 1e-6
    for _ in range(20):
        t, e = rng.integers(q["S"]), rng.integers(q["N"])
        lp, lm = q["lg"].copy(), q["lg"].copy()
        lp[t, e] += h
        lm[t, e] -= h
        assert g[t, e] == pytest.approx((L(lp) - L(lm)) / (2 * h), rel=2e-6, abs=1e-9)
