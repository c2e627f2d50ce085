"""Pins for the oracle's setup stage: smoothing, target pattern, penalty, capacity, cost model.

Nothing here re-types the oracle's formula for c_hat: the pins are the optimality property
that defines c_hat (equal delivery times, no feasible point with a smaller maximum), the two
sum constraints, the homogeneous special case, brute force over integer allocations, and the
measured times of the paper's Table 1.
"""
import itertools
import os

import numpy as np
import pytest

import tamoe_workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_exchange_times.txt")


def _table1():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            rows[key] = np.array([float(v) for v in vals])
    return rows


# ---------------------------------------------------------------------------
# homogeneous network => load-balanced target k*S/N   (Section 4.2, first paragraph)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("P,E,k,S,beta0", [(4, 1, 1, 512, 1.0), (8, 2, 2, 1000, 3.7), (1, 4, 2, 64, 0.2)])
def test_homogeneous_pattern_is_load_balanced(oracle, P, E, k, S, beta0):
    N = P * E
    beta = np.full((P, P), beta0)
    for rank in range(P):
        c_hat = oracle.target_pattern(beta, N, rank, k, S)
        np.testing.assert_allclose(c_hat, k * S / N, rtol=1e-13)
        np.testing.assert_allclose(oracle.penalty(c_hat), 1.0 / N, rtol=1e-13)


# ---------------------------------------------------------------------------
# constraints of the optimisation problem (Section 4.1, the two constraint equations)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", list(W.WORKLOADS))
def test_row_and_column_sums(oracle, name):
    wl = W.WORKLOADS[name]
    beta, level = W.topology(wl)
    rows = np.stack([oracle.target_pattern(beta, wl.N, r, wl.k, wl.S) for r in range(wl.P)])
    # every device sends k*S rows in total, whatever the table
    np.testing.assert_allclose(rows.sum(axis=1), wl.k * wl.S, rtol=1e-12)
    # symmetric tree: every expert receives k*S/E rows in total
    np.testing.assert_allclose(rows.sum(axis=0), wl.k * wl.S / wl.E, rtol=1e-12)
    assert (rows > 0).all()


def test_row_sum_holds_for_any_table(oracle):
    rng = np.random.default_rng(5)
    P, E = 6, 3
    beta = rng.uniform(0.5, 20.0, size=(P, P))
    for rank in (0, 4):
        c_hat = oracle.target_pattern(beta, P * E, rank, 2, 777)
        assert abs(c_hat.sum() - 2 * 777) < 1e-9
        # experts of one device share the device's volume equally
        per_dev = c_hat.reshape(P, E)
        np.testing.assert_allclose(per_dev, per_dev[:, :1].repeat(E, axis=1), rtol=1e-13)


# ---------------------------------------------------------------------------
# optimality: all deliveries of a device take the same time, and no feasible allocation has a
# smaller slowest delivery (the min-max objective of Section 4.1 with the latency dropped)
# ---------------------------------------------------------------------------
def test_equalised_delivery_times_and_volume_linear_in_bandwidth(oracle):
    rng = np.random.default_rng(11)
    P, E, k, S = 5, 2, 2, 300
    N = P * E
    beta = rng.uniform(1.0, 12.0, size=(P, P))
    rank = 3
    c_hat = oracle.target_pattern(beta, N, rank, k, S)
    per_dev = c_hat.reshape(P, E).sum(axis=1)
    times = beta[rank] * per_dev
    np.testing.assert_allclose(times, times[0], rtol=1e-12)
    # "volume linear in bandwidth": c_hat[e] / c_hat[e'] = beta[dev e'] / beta[dev e]
    for e, e2 in [(0, 9), (2, 5), (7, 1)]:
        assert c_hat[e] / c_hat[e2] == pytest.approx(beta[rank, e2 // E] / beta[rank, e // E], rel=1e-12)


def test_no_feasible_perturbation_lowers_the_maximum(oracle):
    rng = np.random.default_rng(2)
    P, k, S = 4, 1, 100
    beta = rng.uniform(1.0, 9.0, size=(P, P))
    c = np.zeros((P, P))
    c[1] = oracle.target_pattern(beta, P, 1, k, S)
    best = oracle.exchange_cost(None, beta, c, 1.0)
    for _ in range(300):
        delta = rng.normal(size=P)
        delta -= delta.mean()                     # keeps the row sum k*S
        trial = c.copy()
        trial[1] = np.maximum(c[1] + 0.5 * delta, 0.0)
        trial[1] *= (k * S) / trial[1].sum()
        assert oracle.exchange_cost(None, beta, trial, 1.0) >= best * (1 - 1e-12)


def test_brute_force_integer_allocations(oracle):
    """Enumerate every way to split 24 rows over 4 destinations; the real-valued target is at
    least as good as the best integer split and lies within one row of it."""
    beta_row = np.array([1.0, 2.0, 7.0, 7.5])
    P, total = 4, 24
    beta = np.tile(beta_row, (P, 1))
    c_hat = oracle.target_pattern(beta, P, 0, 1, total)
    best_cost, best_alloc = None, None
    for a in itertools.product(range(total + 1), repeat=3):
        if sum(a) > total:
            continue
        alloc = np.array(list(a) + [total - sum(a)], dtype=float)
        cost = float((beta_row * alloc).max())
        if best_cost is None or cost < best_cost:
            best_cost, best_alloc = cost, alloc
    relaxed = float((beta_row * c_hat).max())
    assert relaxed <= best_cost + 1e-12
    assert np.abs(best_alloc - c_hat).max() <= 1.0 + 1e-9
    # and the objective function of the oracle agrees with the hand evaluation
    c = np.zeros((P, P))
    c[0] = best_alloc
    assert oracle.exchange_cost(None, beta, c, 1.0) == pytest.approx(best_cost, rel=1e-14)


# ---------------------------------------------------------------------------
# the paper's Table 1 as a worked example of the cost model
# ---------------------------------------------------------------------------
def test_table1_cost_model_predicts_uneven_times(oracle):
    t = _table1()
    total = t["total_mb"][0]
    even_mb = t["ratio_even"] * total
    uneven_mb = t["ratio_uneven"] * total
    beta_row = t["time_even_us"][:4] / even_mb          # us per MB on each of device 0's links
    P = 4
    beta = np.tile(beta_row, (P, 1))
    c_even = np.zeros((P, P)); c_even[0] = even_mb
    c_uneven = np.zeros((P, P)); c_uneven[0] = uneven_mb
    # slowest delivery of the even pattern is the printed maximum by construction
    assert oracle.exchange_cost(None, beta, c_even, 1.0) == pytest.approx(5618.0, rel=1e-12)
    # the linear model predicts the measured slowest delivery of the uneven pattern within 2 %
    pred = oracle.exchange_cost(None, beta, c_uneven, 1.0)
    assert pred == pytest.approx(t["time_uneven_us"][:4].max(), rel=0.02)
    # and uneven beats even, as the paper's measurement shows
    assert pred < 5618.0


def test_table1_target_pattern(oracle):
    """Feed the measured per-link costs to the target pattern: deliveries equalise, the shares
    sum to one, the pattern is far more skewed than the paper's hand-picked 'uneven' split, and
    its slowest delivery is below both printed patterns' slowest delivery."""
    t = _table1()
    beta_row = t["time_even_us"][:4] / 32.0
    beta = np.tile(beta_row, (4, 1))
    c_hat = oracle.target_pattern(beta, 4, 0, 1, 128)    # 128 "rows" of 1 MB
    assert c_hat.sum() == pytest.approx(128.0, rel=1e-13)
    times = beta_row * c_hat
    np.testing.assert_allclose(times, times[0], rtol=1e-12)
    assert times[0] < t["time_uneven_us"][:4].max() < t["time_even_us"][:4].max()
    share = c_hat / 128.0
    assert share[0] > 0.75 and share[2] < 0.03 and share[3] < share[2]
    np.testing.assert_allclose(share, [0.8056, 0.1530, 0.0207, 0.0207], atol=6e-5)


# ---------------------------------------------------------------------------
# two-tier trees: closed forms for the five configurations
# ---------------------------------------------------------------------------
TWO_TIER = {
    # name: (c_hat intra, c_hat inter, penalty intra, penalty inter)
    "tiny": (102.4, 25.6, 0.05, 0.2),
    "small": (8192 / 5.5, 8192 / 44.0, 0.01, 0.08),
    "gpt_moe": (32768 / 13.6, 32768 / 136.0, 1 / 568, 10 / 568),
    "skewed": (16384 / 11.5, 16384 / 184.0, 1 / 904, 16 / 904),
    "large": (131072 / (2 * (8 + 56 / 12)), 131072 / (24 * (8 + 56 / 12)), 1 / 1360, 12 / 1360),
}


@pytest.mark.parametrize("name", list(TWO_TIER))
@pytest.mark.parametrize("rank_sel", ["first", "interior"])
def test_two_tier_closed_form(oracle, name, rank_sel):
    """n nodes x g devices, ratio R: Z = g + (P-g)/R, c_intra = kS/(E Z), c_inter = c_intra/R;
    penalty p_intra = 1/(E (g + (P-g) R)), p_inter = R p_intra."""
    wl = W.WORKLOADS[name]
    rank = 0 if rank_sel == "first" else wl.P // 2 + 1
    beta, level = W.topology(wl)
    c_hat, p, _ = oracle.setup(beta, level, wl.N, rank, wl.k, wl.S, wl.capacity_factor, 0)
    ci, cx, pi, px = TWO_TIER[name]
    node = rank // wl.devs_per_node
    dev_of_e = np.arange(wl.N) // wl.E
    intra = (dev_of_e // wl.devs_per_node) == node
    np.testing.assert_allclose(c_hat[intra], ci, rtol=1e-12)
    np.testing.assert_allclose(c_hat[~intra], cx, rtol=1e-12)
    np.testing.assert_allclose(p[intra], pi, rtol=1e-12)
    np.testing.assert_allclose(p[~intra], px, rtol=1e-12)
    assert p.sum() == pytest.approx(1.0, rel=1e-13)
    assert intra.sum() == wl.devs_per_node * wl.E


def test_penalty_is_normalised_reciprocal(oracle):
    c_hat = np.array([8.0, 4.0, 2.0, 2.0])
    p = oracle.penalty(c_hat)
    assert p.sum() == pytest.approx(1.0)
    # p proportional to 1/c_hat: products p*c_hat all equal
    np.testing.assert_allclose(p * c_hat, (p * c_hat)[0], rtol=1e-14)
    # hand-worked: reciprocals 1/8, 1/4, 1/2, 1/2 sum to 11/8
    np.testing.assert_allclose(p, [1 / 11, 2 / 11, 4 / 11, 4 / 11], rtol=1e-14)


# ---------------------------------------------------------------------------
# capacity
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name,uniform,intra,inter", [
    ("tiny", 64, 103, 26), ("small", 640, 1862, 233), ("gpt_moe", 615, 2892, 290),
    ("skewed", 256, 1425, 90), ("large", 1280, 6468, 539)])
def test_capacity_values(oracle, name, uniform, intra, inter):
    wl = W.WORKLOADS[name]
    beta, level = W.topology(wl)
    _, _, cap0 = oracle.setup(beta, level, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    assert (cap0 == uniform).all()
    _, _, cap1 = oracle.setup(beta, level, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 1)
    n_intra = wl.devs_per_node * wl.E
    assert (cap1[:n_intra] == intra).all() and (cap1[n_intra:] == inter).all()


def test_capacity_exact_products_stay_exact(oracle):
    # 1.0 * 512/8 = 64 exactly; 1.25 * 8192/16 = 640 exactly; 1.2 * 10 = 12 (12.000000000000002 in binary)
    assert (oracle.capacity(np.full(8, 64.0), 1, 512, 1.0, 0) == 64).all()
    assert (oracle.capacity(np.full(4, 10.0), 1, 40, 1.2, 1) == 12).all()
    assert (oracle.capacity(np.full(4, 10.1), 1, 40, 1.0, 1) == 11).all()


# ---------------------------------------------------------------------------
# smoothing per tree level
# ---------------------------------------------------------------------------
def test_smoothing_is_identity_on_noiseless_tree(oracle):
    beta, level = W.two_tier_topology(3, 4, 9.0)
    np.testing.assert_array_equal(oracle.smooth_beta(beta, level), beta)


def test_smoothing_averages_actual_pairs(oracle):
    """[2,2] tree: 2 intra-node pairs (0,1), (2,3) and 4 cross-node pairs; the diagonal carries
    the intra-node label here and therefore takes the intra-node mean."""
    level = np.array([[0, 0, 1, 1], [0, 0, 1, 1], [1, 1, 0, 0], [1, 1, 0, 0]], dtype=np.int32)
    beta = np.array([[0.5, 1.0, 10.0, 12.0],
                     [99.0, 0.5, 14.0, 8.0],
                     [99.0, 99.0, 0.5, 3.0],
                     [99.0, 99.0, 99.0, 0.5]])
    bh = oracle.smooth_beta(beta, level)
    intra = (1.0 + 3.0) / 2
    inter = (10.0 + 12.0 + 14.0 + 8.0) / 4
    expect = np.where(level == 0, intra, inter)
    np.testing.assert_allclose(bh, expect, rtol=1e-15)


def test_smoothing_diagonal_level_of_its_own(oracle):
    level = np.array([[2, 0, 1, 1], [0, 2, 1, 1], [1, 1, 2, 0], [1, 1, 0, 2]], dtype=np.int32)
    beta = np.array([[0.1, 1.0, 5.0, 5.0], [1.0, 0.3, 5.0, 5.0], [5.0, 5.0, 0.2, 2.0], [5.0, 5.0, 2.0, 0.2]])
    bh = oracle.smooth_beta(beta, level)
    assert bh[0, 0] == pytest.approx(0.2) and bh[3, 3] == pytest.approx(0.2)
    assert bh[0, 1] == pytest.approx(1.5) and bh[2, 3] == pytest.approx(1.5)
    assert bh[0, 2] == pytest.approx(5.0)


def test_smoothing_removes_profiling_noise(oracle):
    noisy, level = W.noisy_topology(4, 4, 8.0, seed=9, rel_noise=0.05)
    clean, _ = W.two_tier_topology(4, 4, 8.0)
    bh = oracle.smooth_beta(noisy, level)
    assert len(np.unique(bh)) == 2
    assert np.abs(bh / clean - 1).max() < 0.02 < np.abs(noisy / clean - 1).max()
    # symmetric after smoothing => column constraint holds again
    rows = np.stack([oracle.target_pattern(bh, 16, r, 2, 4096) for r in range(16)])
    np.testing.assert_allclose(rows.sum(axis=0), 2 * 4096, rtol=1e-12)


def test_exchange_cost_takes_the_max_over_all_pairs_and_adds_latency(oracle):
    P, E = 3, 2
    N = P * E
    beta = np.arange(1, 10, dtype=float).reshape(P, P)
    alpha = np.full((P, P), 0.25)
    c = np.arange(P * N, dtype=float).reshape(P, N)
    per_dev = c.reshape(P, P, E).sum(axis=2)
    expect = (alpha + beta * per_dev * 16.0).max()
    assert oracle.exchange_cost(alpha, beta, c, 16.0) == pytest.approx(expect, rel=1e-15)
    assert oracle.exchange_cost(None, beta, c, 16.0) == pytest.approx(expect - 0.25, rel=1e-15)
