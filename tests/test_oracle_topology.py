"""Pins for the oracle's topology front-end: the row problem with the latency term kept (Sections
4.1 / 4.2), ring tables (Section 3.2) and tree topologies in nested-list notation with the merge of
asymmetric trees (Section 4.2)."""
import ast
import itertools
import os

import numpy as np
import pytest

import tamoe_workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---- min-max pattern with latency ---------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "small", "gpt_moe", "large"])
def test_minmax_without_latency_is_the_closed_form(oracle, name):
    wl = W.WORKLOADS[name]
    beta, level = W.topology(wl)
    beta_hat = oracle.smooth_beta(beta, level)
    closed = oracle.target_pattern(beta_hat, wl.N, wl.rank, wl.k, wl.S)
    for alpha in (None, np.zeros(wl.P), np.full(wl.P, 7.5)):          # a common latency shifts T only
        c_hat, T = oracle.minmax_pattern(alpha, beta_hat[wl.rank], wl.N, wl.k, wl.S, 2.0 * wl.d)
        np.testing.assert_allclose(c_hat, closed, rtol=1e-12)
        a0 = 0.0 if alpha is None else alpha[0]
        assert T == pytest.approx(a0 + beta_hat[wl.rank, 0] * 2.0 * wl.d * closed[:wl.E].sum(), rel=1e-12)


def test_minmax_optimality_conditions(oracle):
    rng = np.random.default_rng(1)
    for trial in range(20):
        P, E = int(rng.integers(2, 9)), int(rng.integers(1, 4))
        beta = rng.uniform(0.5, 20.0, size=P)
        alpha = rng.uniform(0.0, 3000.0, size=P) * (trial % 2 + 0.1)
        k, S, bytes_ = 2, 1000, 64.0
        c_hat, T = oracle.minmax_pattern(alpha, beta, P * E, k, S, bytes_)
        v = c_hat.reshape(P, E).sum(axis=1)
        assert (c_hat.reshape(P, E) == c_hat.reshape(P, E)[:, :1]).all()       # experts of a device share equally
        assert v.sum() == pytest.approx(k * S, rel=1e-12)
        cost = alpha + beta * bytes_ * v
        used = v > 0
        np.testing.assert_allclose(cost[used], T, rtol=1e-10)                  # loaded links finish together
        assert (alpha[~used] >= T * (1 - 1e-12)).all()                         # idle links: latency alone is too long
        # the value is what the exchange-cost function says about this pattern (one sender, P receivers)
        full_c = np.zeros((P, P * E))
        full_c[0] = c_hat
        a2 = np.zeros((P, P)); a2[0] = alpha
        b2 = np.full((P, P), 1e-30); b2[0] = beta
        assert oracle.exchange_cost(a2, b2, full_c, bytes_) == pytest.approx(T, rel=1e-10)
        # no feasible pattern is faster: moving rows between any two loaded links raises the slower one
        for a, b in itertools.permutations(np.flatnonzero(used)[:3], 2):
            w = v.copy()
            step = 0.01 * w[a]
            w[a] -= step
            w[b] += step
            assert (alpha + beta * bytes_ * w).max() > T


def test_minmax_brute_force_three_devices(oracle):
    alpha = np.array([0.0, 40.0, 300.0])
    beta = np.array([1.0, 3.0, 2.0])
    k, S, bytes_ = 1, 200, 1.0
    c_hat, T = oracle.minmax_pattern(alpha, beta, 3, k, S, bytes_)
    best = np.inf
    n = 400
    for a in range(n + 1):
        for b in range(n + 1 - a):
            v = np.array([a, b, n - a - b]) * (k * S / n)
            cost = np.where(v > 0, alpha + beta * bytes_ * v, -np.inf).max()
            best = min(best, cost)
    assert T <= best * (1 + 1e-12)
    assert best <= T + beta.max() * bytes_ * (k * S / n) * 2           # the grid gets within two cells of it


def test_minmax_on_the_measured_links_of_table_1(oracle):
    """alpha and beta of the three link types fitted through the two measured points each of the
    paper's Table 1; the optimum of the row problem cannot be slower than either pattern the paper
    measured, and it loads the links in the order of their speed (the row problem has no balance
    constraint across senders, so the local copy, by far the fastest link, takes the most)."""
    rows = {}
    with open(os.path.join(GOLDEN, "table1_exchange_times.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, *vals = line.split()
                rows[key] = [float(v) for v in vals]
    mb = rows["total_mb"][0]
    re_, ru = np.array(rows["ratio_even"]), np.array(rows["ratio_uneven"])
    te, tu = np.array(rows["time_even_us"][:4]), np.array(rows["time_uneven_us"][:4])
    beta = np.empty(4); alpha = np.empty(4)
    for j in range(1, 4):
        beta[j] = (te[j] - tu[j]) / ((re_[j] - ru[j]) * mb)             # us per MB
        alpha[j] = te[j] - beta[j] * re_[j] * mb
    beta[0] = te[0] / (re_[0] * mb); alpha[0] = 0.0                      # self copy: one point only
    assert (beta > 0).all() and (alpha >= 0).all()
    c_hat, T = oracle.minmax_pattern(alpha, beta, 4, 1, int(mb), 1.0)    # unit: one "row" = 1 MB
    assert T < tu[1:].max() < te[1:].max()
    assert c_hat[0] > c_hat[1] > c_hat[2] > 0 and c_hat[1] > c_hat[3] > 0
    assert c_hat[2] < ru[2] * mb and c_hat[3] < ru[3] * mb              # less over the slow tier than "uneven"
    np.testing.assert_allclose(alpha + beta * c_hat, T, rtol=1e-10)
    assert c_hat.sum() == pytest.approx(mb, rel=1e-12)


# ---- ring -----------------------------------------------------------------------------------

def _bottleneck_paths(beta_link):
    """Minimax path over all routes (Floyd-Warshall on the bottleneck semiring)."""
    P = len(beta_link)
    best = np.full((P, P), np.inf)
    for q in range(P):
        a, b = q, (q + 1) % P
        best[a, b] = min(best[a, b], beta_link[q])
        best[b, a] = min(best[b, a], beta_link[q])
    for m in range(P):
        for i in range(P):
            for j in range(P):
                best[i, j] = min(best[i, j], max(best[i, m], best[m, j]))
    return best


def test_ring_uniform_links(oracle):
    P = 8
    beta, alpha, level = oracle.ring_table(np.full(P, 2.0), np.full(P, 5.0), self_beta=0.5, self_alpha=1.0)
    i, j = np.indices((P, P))
    hops = np.minimum((i - j) % P, (j - i) % P)
    np.testing.assert_array_equal(level, hops)
    np.testing.assert_array_equal(beta, np.where(hops == 0, 0.5, 2.0))
    np.testing.assert_array_equal(alpha, np.where(hops == 0, 1.0, 5.0 * hops))


def test_ring_routes_around_a_slow_link_and_matches_minimax_paths(oracle):
    beta, alpha, level = oracle.ring_table([1.0, 1.0, 1.0, 10.0], [1.0, 2.0, 4.0, 8.0])
    assert beta[3, 0] == 1.0 and level[3, 0] == 3 and alpha[3, 0] == 7.0     # 0-1-2-3 instead of the slow link
    assert beta[0, 1] == 1.0 and level[0, 1] == 1 and alpha[0, 1] == 1.0
    rng = np.random.default_rng(2)
    for P in (3, 5, 8, 12):
        links = rng.choice([1.0, 2.0, 6.0], size=P)
        beta, alpha, level = oracle.ring_table(links)
        ref = _bottleneck_paths(links)
        off = ~np.eye(P, dtype=bool)
        np.testing.assert_array_equal(beta[off], ref[off])
        np.testing.assert_array_equal(beta, beta.T)
        np.testing.assert_array_equal(level, level.T)
        assert (level[off] >= 1).all() and (level[off] <= P - 1).all()


# ---- trees ------------------------------------------------------------------------------------

def _levels_by_lists(tree):
    """Independent labelling from the Python literal of the notation."""
    def height(n):
        return 1 if isinstance(n, int) else 1 + max(height(c) for c in n)

    def devices(n):
        return n if isinstance(n, int) else sum(devices(c) for c in n)

    P = devices(tree)
    level = np.zeros((P, P), dtype=np.int32)

    def walk(n, base):
        cnt = devices(n)
        if isinstance(n, int):
            kids = [1] * cnt
        else:
            kids = [devices(c) for c in n]
        starts = np.concatenate([[0], np.cumsum(kids)]) + base
        for a in range(len(kids)):
            for b in range(len(kids)):
                if a != b:
                    level[starts[a]:starts[a + 1], starts[b]:starts[b + 1]] = height(n)
        if not isinstance(n, int):
            for c, s in zip(n, starts):
                walk(c, s)

    walk(tree, 0)
    return level


def test_tree_merge_golden_examples(oracle):
    with open(os.path.join(GOLDEN, "tree_merge_example.txt")) as f:
        cases = [line.split() for line in f if line.strip() and not line.startswith("#")]
    assert len(cases) == 2
    for given, merged in cases:
        lv, text = oracle.tree_levels(given, True)
        assert text == merged
        np.testing.assert_array_equal(lv, _levels_by_lists(ast.literal_eval(merged)))
        lv0, text0 = oracle.tree_levels(given, False)
        assert text0 == given
        np.testing.assert_array_equal(lv0, _levels_by_lists(ast.literal_eval(given)))


def _symmetric(n):
    """Every list's elements are alike, all the way down: the paper's symmetric tree."""
    if isinstance(n, int):
        return True
    return all(_symmetric(c) for c in n) and len({repr(c) for c in n}) == 1


@pytest.mark.parametrize("text", ["8", "[4,4]", "[2,2,2,2]", "[[2,2],[2,2]]", "[[4,4,4],[4,4,4]]", "[[[2,2],[2,2]],[[2,2],[2,2]]]",
                                  "[3,1,2]", "[[2,2],[2]]", "[[2,2],[2,2],[2]]", "[[2],[2,2,2],[2,2,2],[2]]",
                                  "[[[2,2],[2]],[[2,2],[2,2]]]", " [ 2 , [ 3 ] ] ", "[[2,2],[2,2],[2],[2]]",
                                  "[[[2,2],[2,2]],[[2,2]]]", "[[2,2,2],[2],[2,2,2],[2],[2]]"])
def test_tree_levels_invariants(oracle, text):
    plain = ast.literal_eval(text.strip())
    lv, shown = oracle.tree_levels(text, False)
    np.testing.assert_array_equal(lv, _levels_by_lists(plain))
    assert shown == text.replace(" ", "")
    np.testing.assert_array_equal(lv, lv.T)
    assert (np.diag(lv) == 0).all()
    merged_lv, merged, order = oracle.tree_levels(text, True, want_order=True)
    assert merged_lv.shape == lv.shape                                   # devices are neither lost nor made
    tree = ast.literal_eval(merged)
    # devices keep their numbers: the merged tree, read left to right, lists them in `order`
    np.testing.assert_array_equal(np.sort(order), np.arange(lv.shape[0]))
    np.testing.assert_array_equal(merged_lv[np.ix_(order, order)], _levels_by_lists(tree))
    assert (merged_lv <= lv).all()                                       # a merge only brings devices closer
    np.testing.assert_array_equal(oracle.tree_levels(text, False, want_order=True)[2], np.arange(lv.shape[0]))
    if _symmetric(plain):
        assert merged == shown                                           # symmetric trees are left alone
    if _symmetric(tree):
        assert oracle.tree_levels(merged, True)[1] == merged             # nothing left to merge


# The merge rule is this build's reading of one example and one stated aim (Section 4.2, last paragraph:
# a symmetric tree).  Outcomes worked by hand from the rule as the oracle's comment states it (full
# sub-trees = the largest siblings; separate nodes, left to right, go to the least loaded, then nearest,
# then left full sub-tree of their height; one pass from the leaves up).
MERGE_BY_HAND = [
    # given, merged, symmetric afterwards, device numbers in the order of the merged tree (None: unchanged)
    ("[[2,2],[2]]", "[[2,2,2]]", True, None),                            # the paper's example
    ("[[4,4],[4]]", "[[4,4,4]]", True, None),
    ("[[2,2],[2,2],[2],[2]]", "[[2,2,2],[2,2,2]]", True,                 # shared out evenly: the first separate node
     [0, 1, 2, 3, 10, 11, 4, 5, 6, 7, 8, 9]),                            # goes to its neighbour, the second to the other
    ("[[2],[2,2,2],[2,2,2],[2]]", "[[2,2,2,2],[2,2,2,2]]", True,
     [2, 3, 4, 5, 6, 7, 0, 1, 8, 9, 10, 11, 12, 13, 14, 15]),            # members join at the end of the list
    ("[[[2,2],[2,2]],[[2,2]]]", "[[[2,2],[2,2],[2,2]]]", True, None),    # a separate node one layer up
    ("[[2,2,2],[2],[2,2,2],[2],[2]]", "[[2,2,2,2],[2,2,2,2,2]]", False,  # 3 nodes over 2 sub-trees: left (tie),
     None),                                                              # right (less loaded), right (nearer)
    ("[[2,2],[2,2],[2]]", "[[2,2],[2,2,2]]", False, None),               # cannot be shared out: layers are kept
    ("[[[2,2],[2]],[[2,2],[2,2]]]", "[[[2,2],[2,2],[2,2,2]]]", False,    # inner merge first, then one layer up
     [6, 7, 8, 9, 10, 11, 12, 13, 0, 1, 2, 3, 4, 5]),
    ("[3,1,2]", "[3,1,2]", False, None),                                 # device switches are never merged
    ("[[[2,2],[2,2]],[2]]", "[[[2,2],[2,2]],[2]]", False, None),         # no full sub-tree of the node's height
]


@pytest.mark.parametrize("given,merged,sym,order", MERGE_BY_HAND)
def test_tree_merge_rule_by_hand(oracle, given, merged, sym, order):
    lv, text, got_order = oracle.tree_levels(given, True, want_order=True)
    assert text == merged
    assert _symmetric(ast.literal_eval(text)) == sym
    order = np.arange(lv.shape[0]) if order is None else np.array(order)
    np.testing.assert_array_equal(got_order, order)
    np.testing.assert_array_equal(lv[np.ix_(order, order)], _levels_by_lists(ast.literal_eval(merged)))


@pytest.mark.parametrize("given,merged,sym,order", MERGE_BY_HAND)
def test_tree_merge_restores_the_receive_constraint_where_it_makes_the_tree_symmetric(oracle, given, merged, sym, order):
    """What the merge is for (Section 4.2: optimise "as the symmetric structure"): on a symmetric tree
    every device sees the same set of link levels, so the closed-form pattern of all senders together
    gives every expert k*S/E rows (the second constraint of Section 4.1).  Where the rule cannot make
    the tree symmetric the constraint stays violated, and the hierarchy is kept instead of being
    flattened into one switch."""
    lv, text = oracle.tree_levels(given, True)
    P = lv.shape[0]
    E, k, S = 2, 2, 1000
    N = P * E
    per_level = np.array([1.0, 1.0, 3.0, 10.0, 31.0])                    # self, same switch, one up, ...
    beta_hat = per_level[lv]
    c = np.stack([oracle.target_pattern(beta_hat, N, i, k, S) for i in range(P)])
    np.testing.assert_allclose(c.sum(axis=1), k * S, rtol=1e-12)         # first constraint: always
    col = c.sum(axis=0)
    seen = {tuple(sorted(row)) for row in lv.tolist()}
    if sym:
        assert len(seen) == 1
        np.testing.assert_allclose(col, k * S * P / N, rtol=1e-12)
    else:
        assert len(seen) > 1
        assert np.abs(col / (k * S * P / N) - 1.0).max() > 1e-3
    if given == "[[2,2],[2,2],[2]]":
        assert lv.max() == 3                                             # still three layers, not one flat switch
        lv0, _ = oracle.tree_levels(given, False)
        c0 = np.stack([oracle.target_pattern(per_level[lv0], N, i, k, S) for i in range(P)])
        spread = lambda v: v.max() / v.min()
        assert spread(col) < spread(c0.sum(axis=0))                      # and the isolated node is better served


def test_tree_two_tier_levels_give_the_generator_table(oracle):
    lv, _ = oracle.tree_levels("[4,4,4,4]", False)
    _, level = W.two_tier_topology(4, 4, 8.0)
    np.testing.assert_array_equal((lv == 2), level == 1)                 # same partition into tiers
    beta, _ = W.noisy_topology(4, 4, 8.0, seed=3)
    np.testing.assert_allclose(oracle.smooth_beta(beta, lv), oracle.smooth_beta(beta, level + np.eye(16, dtype=np.int32) * 0),
                               rtol=0.06)


@pytest.mark.parametrize("bad", ["", "[", "[2,", "[2,,2]", "[]", "[0]", "[2]]", "[a]", "2,2"])
def test_tree_rejects_bad_text(oracle, bad):
    with pytest.raises(ValueError):
        oracle.tree_levels(bad, False)
