"""Pins for the oracle's gate stage: scores, softmax, top-k, load statistics and the two losses.

Library routines (numpy matmul, scipy softmax, numpy stable argsort / bincount) and pure-Python
brute force serve as independent references; closed forms pin the losses.
"""
import math

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import tamoe_workloads as W


# ---------------------------------------------------------------------------
# storage rounding used by the oracle's outputs
# ---------------------------------------------------------------------------
def test_bf16_rounding_matches_bit_trick_on_float32_values(oracle):
    rng = np.random.default_rng(0)
    vals = np.concatenate([
        rng.standard_normal(4000).astype(np.float32),
        (rng.standard_normal(500) * 1e-30).astype(np.float32),
        (rng.standard_normal(500) * 1e30).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40, -1e-40], dtype=np.float32),
    ])
    expect = W.f32_to_bf16_bits(vals)
    got = np.array([oracle.round_to_bf16(float(v)) for v in vals], dtype=np.uint16)
    np.testing.assert_array_equal(got, expect)


def test_bf16_rounding_is_single_rounding_from_double(oracle):
    # 1 + 2^-8 is a tie between 1.0 (0x3F80) and 1 + 2^-7 (0x3F81): ties go to even
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert oracle.round_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # a hair above the tie must round up; rounding through float32 first would lose the hair
    assert oracle.round_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle.round_to_bf16(-(1.0 + 2.0 ** -8 + 2.0 ** -40)) == 0xBF81
    assert oracle.round_to_bf16(float("inf")) == 0x7F80
    assert oracle.round_to_bf16(1e39) == 0x7F80


# ---------------------------------------------------------------------------
# scores: textbook matrix product
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,S,d,N", [(W.F32, 37, 24, 5), (W.BF16, 65, 40, 12)])
def test_logits_equal_matmul(oracle, dtype, S, d, N):
    rng = np.random.default_rng(3)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    w = W.to_storage(rng.standard_normal((N, d)).astype(np.float32), dtype)
    ref = W.storage_to_f64(x, dtype) @ W.storage_to_f64(w, dtype).T
    got = oracle.logits(x, w, dtype)
    assert got.shape == (S, N)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-12)


def test_logits_basis_vectors(oracle):
    """x = unit vectors picks out columns of W: catches a transposed or mis-strided operand."""
    d, N = 6, 4
    w = np.arange(N * d, dtype=np.float32).reshape(N, d)
    x = np.eye(d, dtype=np.float32)
    got = oracle.logits(x, w, W.F32)
    np.testing.assert_array_equal(got, w.T.astype(np.float64))


def test_threads_do_not_change_results(oracle):
    wl = W.WORKLOADS["tiny"]
    inp = W.make_inputs(wl)
    oracle.set_threads(1)
    a = oracle.logits(inp["x"], inp["w"], wl.dtype)
    oracle.set_threads(4)
    b = oracle.logits(inp["x"], inp["w"], wl.dtype)
    oracle.set_threads(1)
    np.testing.assert_array_equal(a, b)


# ---------------------------------------------------------------------------
# softmax and top-k
# ---------------------------------------------------------------------------
def test_softmax_matches_scipy_and_is_shift_invariant(oracle):
    lg = W.random_logits(1, 200, 17).astype(np.float64) * 3
    G = oracle.softmax(lg)
    np.testing.assert_allclose(G, scipy_softmax(lg, axis=1), rtol=1e-13)
    np.testing.assert_allclose(G.sum(axis=1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(oracle.softmax(lg + 1000.0), G, rtol=1e-10)   # no overflow either
    assert np.isfinite(oracle.softmax(lg * 500)).all()


@pytest.mark.parametrize("k", [1, 2, 3, 8])
def test_topk_matches_stable_argsort(oracle, k):
    lg = W.random_logits(2, 300, 8).astype(np.float64)
    G = oracle.softmax(lg)
    idx, wgt = oracle.topk(lg, G, k)
    ref = np.argsort(-lg, axis=1, kind="stable")[:, :k]
    np.testing.assert_array_equal(idx, ref)
    np.testing.assert_array_equal(wgt, np.take_along_axis(G, ref, axis=1))
    # distinct experts, scores non-increasing
    assert all(len(set(r)) == k for r in idx)
    sel = np.take_along_axis(lg, idx, axis=1)
    assert (np.diff(sel, axis=1) <= 0).all()


def test_topk_ties_go_to_lowest_index(oracle):
    lg = np.zeros((3, 6))
    lg[1] = [1, 5, 5, 0, 5, 1]
    lg[2] = [2, 2, 3, 3, 1, 1]
    G = oracle.softmax(lg)
    idx, _ = oracle.topk(lg, G, 4)
    np.testing.assert_array_equal(idx[0], [0, 1, 2, 3])
    np.testing.assert_array_equal(idx[1], [1, 2, 4, 0])
    np.testing.assert_array_equal(idx[2], [2, 3, 0, 1])
    # many ties, against the stable sort
    lt = W.random_logits(4, 500, 16, ties=True).astype(np.float64)
    idx, _ = oracle.topk(lt, oracle.softmax(lt), 3)
    np.testing.assert_array_equal(idx, np.argsort(-lt, axis=1, kind="stable")[:, :3])


def test_topk_weights_are_raw_softmax_values(oracle):
    lg = np.log(np.array([[0.5, 0.3, 0.2], [0.1, 0.2, 0.7]]))
    idx, wgt = oracle.topk(lg, oracle.softmax(lg), 2)
    np.testing.assert_array_equal(idx, [[0, 1], [2, 1]])
    np.testing.assert_allclose(wgt, [[0.5, 0.3], [0.7, 0.2]], rtol=1e-14)   # not renormalised to 1


# ---------------------------------------------------------------------------
# load statistics
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("P,E,k", [(4, 1, 1), (4, 2, 2), (2, 3, 3)])
def test_counts(oracle, P, E, k):
    N, S = P * E, 333
    lg = W.random_logits(7, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    idx, _ = oracle.topk(lg, G, k)
    c_e, c_d, m = oracle.counts(idx, G, P)
    np.testing.assert_array_equal(c_e, np.bincount(idx.ravel(), minlength=N))
    np.testing.assert_array_equal(c_d, c_e.reshape(P, E).sum(axis=1))
    assert c_e.sum() == k * S and c_d.sum() == k * S
    np.testing.assert_allclose(m, G.mean(axis=0), rtol=1e-13)
    assert m.sum() == pytest.approx(1.0, rel=1e-13)


# ---------------------------------------------------------------------------
# losses: closed forms
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny", "small", "large"])
def test_uniform_routing_any_topology(oracle, name):
    """m = 1/N, c = kS/N  =>  l_aux = k/N and l_topo = k*P/N = k/E, whatever the table."""
    wl = W.WORKLOADS[name]
    beta, level = W.topology(wl)
    _, p, _ = oracle.setup(beta, level, wl.N, wl.P // 2 + 1, wl.k, wl.S, wl.capacity_factor, 0)
    m = np.full(wl.N, 1.0 / wl.N)
    c = np.full(wl.N, wl.k * wl.S // wl.N, dtype=np.int32)
    assert oracle.l_aux(m, c, wl.S) == pytest.approx(wl.k / wl.N, rel=1e-13)
    assert oracle.l_topo(p, m, c, wl.P, wl.S) == pytest.approx(wl.k / wl.E, rel=1e-13)


def test_uniform_topology_any_routing(oracle):
    """Homogeneous table => p = 1/N => l_topo = P * l_aux for arbitrary routing."""
    P, E, k, S = 4, 2, 2, 257
    N = P * E
    lg = W.random_logits(8, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    idx, _ = oracle.topk(lg, G, k)
    c_e, _, m = oracle.counts(idx, G, P)
    p = oracle.penalty(oracle.target_pattern(np.full((P, P), 2.5), N, 1, k, S))
    la = oracle.l_aux(m, c_e, S)
    assert oracle.l_topo(p, m, c_e, P, S) == pytest.approx(P * la, rel=1e-13)
    assert la == pytest.approx(float((m * c_e).sum() / S), rel=1e-13)


def test_routing_at_target(oracle):
    """c = c_hat (integers here) and m = c_hat/(kS): every term p*m*c is equal, so
    l_topo = N*P / (S * sum_e 1/c_hat[e])."""
    nodes, g, R, k, S = 2, 2, 4.0, 1, 500
    P = N = 4
    beta, _ = W.two_tier_topology(nodes, g, R)
    c_hat = oracle.target_pattern(beta, N, 0, k, S)        # 200, 200, 50, 50
    np.testing.assert_allclose(c_hat, [200, 200, 50, 50], rtol=1e-13)
    p = oracle.penalty(c_hat)
    m = c_hat / (k * S)
    c = c_hat.astype(np.int32)
    assert oracle.l_topo(p, m, c, P, S) == pytest.approx(N * P / (S * (1.0 / c_hat).sum()), rel=1e-13)
    # hand value: p = (.1,.1,.4,.4); sum p m c = 2*(.1*.4*200) + 2*(.4*.1*50) = 20; 16*20/500
    assert oracle.l_topo(p, m, c, P, S) == pytest.approx(0.64, rel=1e-13)


def test_loss_penalises_slow_links_more(oracle):
    """Moving load from a fast-link expert to a slow-link expert raises l_topo but not l_aux's
    symmetric counterpart: the reweighting is what carries the topology."""
    beta, _ = W.two_tier_topology(2, 2, 4.0)
    p = oracle.penalty(oracle.target_pattern(beta, 4, 0, 1, 400))
    m = np.full(4, 0.25)
    near = np.array([160, 160, 40, 40], dtype=np.int32)
    far = np.array([40, 40, 160, 160], dtype=np.int32)
    assert oracle.l_aux(m, near, 400) == pytest.approx(oracle.l_aux(m, far, 400))
    assert oracle.l_topo(p, m, far, 4, 400) > 2.0 * oracle.l_topo(p, m, near, 4, 400)


# ---------------------------------------------------------------------------
# brute force on tiny inputs: the whole gate stage in pure Python
# ---------------------------------------------------------------------------
def _brute_gate(lg, k, P, p):
    S, N = len(lg), len(lg[0])
    E = N // P
    c = [0] * N
    msum = [0.0] * N
    chosen = []
    for t in range(S):
        mx = max(lg[t])
        ex = [math.exp(v - mx) for v in lg[t]]
        den = math.fsum(ex)
        g = [v / den for v in ex]
        order = sorted(range(N), key=lambda e: (-lg[t][e], e))[:k]
        chosen.append([(e, g[e]) for e in order])
        for e in order:
            c[e] += 1
        for e in range(N):
            msum[e] += g[e]
    m = [v / S for v in msum]
    l_aux = math.fsum(m[e] * c[e] / S for e in range(N))
    l_topo = N * P * math.fsum(p[e] * m[e] * c[e] / S for e in range(N))
    c_dev = [sum(c[j * E:(j + 1) * E]) for j in range(P)]
    return chosen, c, c_dev, m, l_aux, l_topo


@pytest.mark.parametrize("S,P,E,k,seed", [(8, 2, 2, 2, 0), (7, 4, 1, 1, 1), (5, 1, 3, 3, 2), (8, 2, 1, 2, 3)])
def test_brute_force_gate(oracle, S, P, E, k, seed):
    N = P * E
    lg = W.random_logits(seed, S, N, ties=(seed % 2 == 1)).astype(np.float64)
    beta, _ = W.two_tier_topology(P, 1, 5.0) if P > 1 else (np.ones((1, 1)), None)
    rank = P - 1
    p = oracle.penalty(oracle.target_pattern(beta, N, rank, k, S))
    r = oracle.route_from_logits(lg, k, P, p, np.full(N, S * k, dtype=np.int32))
    chosen, c, c_dev, m, la, lt = _brute_gate(lg.tolist(), k, P, p.tolist())
    np.testing.assert_array_equal(r["topk_idx"], [[e for e, _ in row] for row in chosen])
    np.testing.assert_allclose(r["topk_w"], [[g for _, g in row] for row in chosen], rtol=1e-13)
    np.testing.assert_array_equal(r["c_expert"], c)
    np.testing.assert_array_equal(r["c_device"], c_dev)
    np.testing.assert_allclose(r["m"], m, rtol=1e-13)
    assert r["l_aux"] == pytest.approx(la, rel=1e-13)
    assert r["l_topo"] == pytest.approx(lt, rel=1e-13)
