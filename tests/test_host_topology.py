"""The library's host-side topology front-end (tamoe_tree_levels, tamoe_ring_table,
tamoe_minmax_pattern) against the oracle, which solves the same problems by other means (bisection
instead of the sorted-prefix solve, overwrite labelling instead of ancestor chains), and its
argument checks.  No GPU is involved."""
import os

import numpy as np
import pytest

import tamoe_workloads as W


@pytest.fixture(scope="module")
def T():
    import paper_2302_09915_amd as T

    if not os.path.exists(T.LIB_PATH):
        from paper_2302_09915_amd import build

        build.build()
    T.lib()
    return T


TREES = ["8", "[4,4]", "[2,2,2,2]", "[[2,2],[2,2]]", "[[4,4,4],[4,4,4]]", "[[[2,2],[2,2]],[[2,2],[2,2]]]", "[3,1,2]",
         "[[2,2],[2]]", "[[2,2],[2,2],[2]]", "[[2],[2,2,2],[2,2,2],[2]]", "[[[2,2],[2]],[[2,2],[2,2]]]", "[2,[3]]",
         " [ 2 , [ 3 ] ] ", "[[8,8,8,8,8,8,8,8]]", "[[1],[1,1],[1,1,1]]", "[[2,[2]],[2]]", "[[2,2],[2,2],[2],[2]]",
         "[[[2,2],[2,2]],[[2,2]]]", "[[2,2,2],[2],[2,2,2],[2],[2]]", "[[[2,2],[2,2]],[2]]", "[[4,4],[4]]",
         "[[3],[3,3],[3],[3,3],[3],[3,3],[3]]", "[[[2],[2,2]],[[2,2],[2]],[[2]]]"]


@pytest.mark.parametrize("text", TREES)
@pytest.mark.parametrize("merge", [False, True])
def test_tree_levels_match_oracle(T, oracle, text, merge):
    lv, shown, order = T.tamoe_tree_levels(text, merge, want_order=True)
    ref_lv, ref_shown, ref_order = oracle.tree_levels(text, merge, want_order=True)
    assert shown == ref_shown
    np.testing.assert_array_equal(lv, ref_lv)
    np.testing.assert_array_equal(order, ref_order)


def test_tree_levels_feed_the_pattern(T, oracle):
    """[8,8,...] x 8 with merge off is the benchmark's two-tier topology: same smoothed pattern."""
    wl = W.WORKLOADS["gpt_moe"]
    lv, _ = T.tamoe_tree_levels("[" + ",".join(["8"] * 8) + "]", False)
    beta, level = W.topology(wl)
    a = T.tamoe_topo_pattern(beta, lv, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 1)
    b = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 1)
    for u, v in zip(a, b):
        np.testing.assert_array_equal(u, v)


@pytest.mark.parametrize("bad", ["", "[", "[2,", "[2,,2]", "[]", "[0]", "[2]]", "[a]", "2,2", "[99999999999]"])
def test_tree_levels_reject_bad_text(T, bad):
    with pytest.raises(T.TamoeError) as ei:
        T.tamoe_tree_levels(bad, False)
    assert ei.value.status == T.INVALID_ARG and "tamoe_tree_levels" in ei.value.message


def test_tree_levels_reject_a_table_that_is_too_small(T):
    with pytest.raises(T.TamoeError) as ei:
        T.tamoe_tree_levels("[4,4]", False, max_P=7)
    assert "8 devices" in ei.value.message


def test_ring_table_matches_oracle(T, oracle):
    rng = np.random.default_rng(5)
    for P in (2, 3, 4, 7, 8, 16):
        for with_alpha in (False, True):
            bl = rng.choice([1.0, 2.0, 6.0, 6.5], size=P)
            al = rng.uniform(0.0, 4.0, size=P) if with_alpha else None
            got = T.tamoe_ring_table(bl, al, 0.25, 0.5)
            ref = oracle.ring_table(bl, al, 0.25, 0.5)
            np.testing.assert_array_equal(got[0], ref[0])
            np.testing.assert_array_equal(got[2], ref[2])
            np.testing.assert_allclose(got[1], ref[1], rtol=1e-15, atol=0)     # sums taken in the same link order


def test_ring_table_rejects_bad_arguments(T):
    for bl, al, sb in (([1.0], None, 1.0), ([1.0, 0.0], None, 1.0), ([1.0, 2.0], [0.0, -1.0], 1.0),
                       ([1.0, 2.0], None, 0.0), ([1.0, float("nan")], None, 1.0)):
        with pytest.raises(T.TamoeError) as ei:
            T.tamoe_ring_table(bl, al, sb)
        assert ei.value.status == T.INVALID_ARG


def test_minmax_pattern_matches_oracle_and_the_closed_form(T, oracle):
    rng = np.random.default_rng(6)
    for trial in range(40):
        P, E = int(rng.integers(1, 17)), int(rng.integers(1, 4))
        beta = rng.uniform(0.5, 20.0, size=P)
        alpha = None if trial % 4 == 0 else rng.uniform(0.0, 5000.0, size=P) * (trial % 3)
        k, S, bytes_ = int(rng.integers(1, 3)), int(rng.integers(1, 5000)), float(rng.choice([1.0, 128.0, 8192.0]))
        c_hat, t = T.tamoe_minmax_pattern(alpha, beta, P * E, k, S, bytes_)
        ref_c, ref_t = oracle.minmax_pattern(alpha, beta, P * E, k, S, bytes_)
        np.testing.assert_allclose(c_hat, ref_c, rtol=1e-9, atol=1e-9 * k * S)
        assert t == pytest.approx(ref_t, rel=1e-12)
    for name in ("tiny", "large"):
        wl = W.WORKLOADS[name]
        beta, level = W.topology(wl)
        c_ref, _, _ = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor, 0)
        beta_hat = oracle.smooth_beta(beta, level)
        c_hat, _ = T.tamoe_minmax_pattern(None, beta_hat[wl.rank], wl.N, wl.k, wl.S, 2.0 * wl.d)
        np.testing.assert_allclose(c_hat, c_ref, rtol=1e-13)


def test_what_dropping_the_latency_costs(T, oracle):
    """The closed form ignores alpha; evaluated with alpha it is never faster than the exact optimum, and
    the two agree when the latencies are small against the transfer times."""
    wl = W.WORKLOADS["gpt_moe"]
    beta, level = W.topology(wl)
    beta_row = oracle.smooth_beta(beta, level)[0] * 1e-4                     # us per byte
    bytes_ = 2.0 * wl.d
    closed, _ = T.tamoe_minmax_pattern(None, beta_row, wl.N, wl.k, wl.S, bytes_)
    for scale, close in ((1e-3, True), (50.0, False)):
        alpha_row = np.where(np.arange(wl.P) < 8, 1.0, 20.0) * scale
        exact, t_exact = T.tamoe_minmax_pattern(alpha_row, beta_row, wl.N, wl.k, wl.S, bytes_)
        t_closed = (alpha_row + beta_row * bytes_ * closed.reshape(wl.P, -1).sum(axis=1)).max()
        assert t_closed >= t_exact * (1 - 1e-12)
        assert (t_closed / t_exact < 1.001) == close


def test_minmax_pattern_rejects_bad_arguments(T):
    ok = dict(alpha_row=None, beta_row=[1.0, 2.0], N=4, k=1, S=10, bytes_per_row=2.0)
    T.tamoe_minmax_pattern(**ok)
    for bad in (dict(N=3), dict(k=0), dict(S=0), dict(bytes_per_row=0.0), dict(beta_row=[1.0, -2.0]),
                dict(alpha_row=[0.0, float("inf")]), dict(alpha_row=[-1.0, 0.0])):
        with pytest.raises(T.TamoeError) as ei:
            T.tamoe_minmax_pattern(**dict(ok, **bad))
        assert ei.value.status == T.INVALID_ARG, bad
