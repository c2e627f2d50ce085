"""Pins for the oracle's receive-side regrouping: brute force by concatenation, the inverse, and
the cases where it is the identity."""
import numpy as np
import pytest

import tamoe_workloads as W


def _brute(rows, cnt):
    P, E = cnt.shape
    seg, pos = {}, 0
    for s in range(P):
        for e in range(E):
            seg[(s, e)] = rows[pos:pos + cnt[s, e]]
            pos += cnt[s, e]
    parts = [seg[(s, e)] for e in range(E) for s in range(P)]
    out = np.concatenate(parts) if parts else rows[:0]
    eoff = np.concatenate([[0], np.cumsum(cnt.sum(axis=0))])
    return out, eoff


@pytest.mark.parametrize("P,E,dtype", [(4, 2, W.F32), (3, 5, W.BF16), (8, 1, W.BF16), (1, 4, W.F32), (5, 3, W.F32)])
def test_regroup_matches_concatenation_and_inverts(oracle, P, E, dtype):
    rng = np.random.default_rng(P * 10 + E)
    cnt = rng.integers(0, 7, size=(P, E)).astype(np.int32)
    cnt[rng.integers(P), rng.integers(E)] = 0                  # an empty segment
    R, d = int(cnt.sum()), 8
    rows = W.to_storage(rng.standard_normal((R, d)).astype(np.float32), dtype)
    out, eoff = oracle.regroup(rows, dtype, cnt, True)
    bo, be = _brute(rows, cnt)
    np.testing.assert_array_equal(out, bo)
    np.testing.assert_array_equal(eoff, be)
    back, _ = oracle.regroup(out, dtype, cnt, False)
    np.testing.assert_array_equal(back, rows)
    if E == 1 or P == 1:
        np.testing.assert_array_equal(out, rows)               # one expert per device: nothing moves


def test_regroup_rows_of_an_expert_keep_source_order(oracle):
    cnt = np.array([[2, 1], [1, 2]], dtype=np.int32)           # P = 2, E = 2
    rows = np.arange(6, dtype=np.float32).reshape(6, 1).repeat(4, axis=1)
    out, eoff = oracle.regroup(rows, W.F32, cnt, True)
    # source-major: s0e0 = rows 0,1; s0e1 = 2; s1e0 = 3; s1e1 = 4,5  ->  expert 0: 0,1,3; expert 1: 2,4,5
    np.testing.assert_array_equal(out[:, 0], [0, 1, 3, 2, 4, 5])
    np.testing.assert_array_equal(eoff, [0, 3, 6])
