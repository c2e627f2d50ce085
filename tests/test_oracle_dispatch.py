"""Pins for the oracle's capacity-limited slot assignment, scatter and combine."""
import numpy as np
import pytest

import tamoe_workloads as W


def _brute_slots(idx, cap, P):
    """Stable sort of the pairs by (expert, choice, token); rank inside the expert = position."""
    S, k = idx.shape
    N = len(cap)
    E = N // P
    pairs = sorted((int(idx[t, j]), j, t) for t in range(S) for j in range(k))
    slot = -np.ones((S, k), dtype=np.int64)
    kept = [0] * N
    rank_in_e = {}
    for e, j, t in pairs:
        r = rank_in_e.get(e, 0)
        rank_in_e[e] = r + 1
        if r < cap[e]:
            kept[e] += 1
    off = np.concatenate([[0], np.cumsum(kept)])
    rank_in_e = {}
    for e, j, t in pairs:
        r = rank_in_e.get(e, 0)
        rank_in_e[e] = r + 1
        if r < cap[e]:
            slot[t, j] = off[e] + r
    scd = [sum(kept[j * E:(j + 1) * E]) for j in range(P)]
    return slot, np.array(kept), off, np.array(scd)


@pytest.mark.parametrize("S,P,E,k,capv,skew", [
    (64, 4, 1, 1, 16, 0.0), (50, 2, 2, 2, 9, 1.0), (33, 1, 4, 3, 1000, 0.5), (40, 4, 2, 2, 0, 0.0),
    (97, 3, 2, 2, 7, 2.0)])
def test_slots_match_brute_force(oracle, S, P, E, k, capv, skew):
    N = P * E
    idx = W.random_routing(S + k, S, N, k, skew)
    cap = np.full(N, capv, dtype=np.int32)
    if capv > 0:
        cap[::2] += 3          # non-uniform capacities
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    bs, bk, bo, bd = _brute_slots(idx, cap, P)
    np.testing.assert_array_equal(slot, bs)
    np.testing.assert_array_equal(kept, bk)
    np.testing.assert_array_equal(off, bo)
    np.testing.assert_array_equal(scd, bd)
    assert K == bo[-1]


def test_slot_invariants(oracle):
    S, P, E, k = 2000, 4, 2, 2
    N = P * E
    idx = W.random_routing(3, S, N, k, skew=1.5)
    cap = np.full(N, 300, dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    c = np.bincount(idx.ravel(), minlength=N)
    np.testing.assert_array_equal(kept, np.minimum(c, cap))
    assert (kept < c).any(), "test needs drops"
    live = slot[slot >= 0]
    assert len(live) == K == kept.sum()
    np.testing.assert_array_equal(np.sort(live), np.arange(K))       # a permutation of 0..K-1
    assert scd.sum() == K
    for e in range(N):
        s_e = slot[idx == e]
        kept_e = s_e[s_e >= 0]
        assert len(kept_e) == kept[e] and (kept_e >= off[e]).all() and (kept_e < off[e] + cap[e]).all()
    # priority: every first choice of an expert comes before any second choice of it, and inside
    # one choice earlier tokens come first
    for e in range(N):
        for j in range(k):
            t_sel = np.nonzero(idx[:, j] == e)[0]
            s = slot[t_sel, j]
            pos = np.where(s >= 0, s, np.iinfo(np.int32).max)
            assert (np.diff(pos) >= 0).all()
        first = slot[idx[:, 0] == e, 0]
        second = slot[idx[:, 1] == e, 1]
        if (second >= 0).any():
            assert (first >= 0).all() and first.max() < second[second >= 0].min()


def test_dropped_first_choice_does_not_affect_second(oracle):
    # tokens 0,1,2 all choose expert 0 first (cap 2 -> token 2 dropped), expert 1 second
    idx = np.array([[0, 1], [0, 1], [0, 1]], dtype=np.int32)
    cap = np.array([2, 5], dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, 1)
    np.testing.assert_array_equal(slot, [[0, 2], [1, 3], [-1, 4]])
    np.testing.assert_array_equal(kept, [2, 3])
    np.testing.assert_array_equal(off, [0, 2, 5])
    assert K == 5 and scd[0] == 5


def test_empty_expert_and_zero_capacity(oracle):
    idx = np.array([[2], [2], [0]], dtype=np.int32)
    cap = np.array([1, 4, 0, 4], dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, 2)
    np.testing.assert_array_equal(slot, [[-1], [-1], [0]])
    np.testing.assert_array_equal(kept, [1, 0, 0, 0])
    np.testing.assert_array_equal(scd, [1, 0])
    assert K == 1


# ---------------------------------------------------------------------------
# scatter and combine
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_scatter_is_a_bit_copy_grouped_by_expert(oracle, dtype):
    S, d, P, E, k = 120, 24, 2, 2, 2
    N = P * E
    rng = np.random.default_rng(4)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    idx = W.random_routing(11, S, N, k, skew=1.0)
    cap = np.full(N, 40, dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    send = oracle.scatter(x, dtype, slot, K)
    assert send.shape == (K, d) and send.dtype == x.dtype
    owner = -np.ones(K, dtype=np.int64)
    for t in range(S):
        for j in range(k):
            if slot[t, j] >= 0:
                np.testing.assert_array_equal(send[slot[t, j]], x[t])
                owner[slot[t, j]] = idx[t, j]
    # rows are listed expert by expert, ascending
    assert (np.diff(owner) >= 0).all()
    np.testing.assert_array_equal(np.bincount(owner, minlength=N), kept)


@pytest.mark.parametrize("dtype", [W.F32, W.BF16])
def test_identity_expert_round_trip(oracle, dtype):
    """recv = send  =>  y[t] = (sum of the weights of the kept choices) * x[t]."""
    S, d, P, E, k = 90, 16, 4, 1, 2
    N = P * E
    rng = np.random.default_rng(6)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    lg = W.random_logits(12, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    idx, wgt = oracle.topk(lg, G, k)
    cap = np.full(N, 30, dtype=np.int32)
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    assert (slot < 0).any()
    send = oracle.scatter(x, dtype, slot, K)
    y_exact, y = oracle.combine(send, dtype, slot, wgt)
    wsum = np.where(slot >= 0, wgt, 0.0).sum(axis=1)
    xv = W.storage_to_f64(x, dtype)
    np.testing.assert_allclose(y_exact, wsum[:, None] * xv, rtol=1e-13, atol=1e-300)
    # fully dropped tokens give a zero row
    dead = (slot < 0).all(axis=1)
    if dead.any():
        assert (y_exact[dead] == 0).all()
    # rounded output: float32 cast, or single rounding to bf16 (checked against the bit trick on
    # values that are exactly float32: use power-of-two weights for that)
    if dtype == W.F32:
        np.testing.assert_array_equal(y, y_exact.astype(np.float32))
    w2 = np.where(wgt > 0.3, 0.5, 0.25)
    ye2, y2 = oracle.combine(send, dtype, slot, w2)
    if dtype == W.BF16:
        np.testing.assert_array_equal(y2, W.f32_to_bf16_bits(ye2.astype(np.float32)))


def test_all_experts_selected_reproduces_input(oracle):
    """k = N, no drops: the weights of a token sum to one, so y = x up to rounding."""
    S, d, N = 40, 8, 4
    rng = np.random.default_rng(8)
    x = rng.standard_normal((S, d)).astype(np.float32)
    lg = W.random_logits(13, S, N).astype(np.float64)
    G = oracle.softmax(lg)
    idx, wgt = oracle.topk(lg, G, N)
    slot, kept, off, scd, K = oracle.slots(idx, np.full(N, S, dtype=np.int32), 2)
    assert K == S * N
    send = oracle.scatter(x, W.F32, slot, K)
    y_exact, _ = oracle.combine(send, W.F32, slot, wgt)
    np.testing.assert_allclose(y_exact, x.astype(np.float64), rtol=1e-12)


def test_combine_uses_the_row_the_slot_names(oracle):
    """Distinct recv rows (not the identity expert): hand-checkable weighted sum."""
    recv = np.array([[1, 10], [2, 20], [3, 30]], dtype=np.float32)
    slot = np.array([[2, 0], [-1, 1], [-1, -1]], dtype=np.int32)
    wgt = np.array([[0.5, 0.25], [0.9, 0.1], [0.6, 0.4]])
    y_exact, y = oracle.combine(recv, W.F32, slot, wgt)
    np.testing.assert_allclose(y_exact, [[1.75, 17.5], [0.2, 2.0], [0.0, 0.0]], rtol=1e-15)
    np.testing.assert_array_equal(y, y_exact.astype(np.float32))


def test_whole_path_invariants_on_tiny_config(oracle):
    wl = W.WORKLOADS["tiny"]
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    c_hat, p, cap = oracle.setup(beta, level, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor, 0)
    lg = oracle.logits(inp["x"], inp["w"], wl.dtype)
    r = oracle.route_from_logits(lg, wl.k, wl.P, p, cap)
    assert r["c_expert"].sum() == wl.k * wl.S
    assert (r["kept"] <= cap).all() and r["K"] == r["kept"].sum()
    live = r["slot"][r["slot"] >= 0]
    np.testing.assert_array_equal(np.sort(live), np.arange(r["K"]))
    # close to uniform routing => loss close to its uniform-routing value k/E = 1
    assert 0.9 < r["l_topo"] < 1.2
