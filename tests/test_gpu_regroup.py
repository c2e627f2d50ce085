"""Parity of tamoe_regroup (receive-side regrouping per local expert) against the oracle: a pure
row permutation, so everything is bit-exact."""
import numpy as np
import pytest

import tamoe_workloads as W
from test_gpu_parity import to_dev, to_host

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU")
    import paper_2302_09915_amd as T

    T.lib()
    return T


@pytest.mark.parametrize("P,E,d,dtype,mean_rows", [
    (64, 2, 4096, W.BF16, 40), (8, 1, 64, W.F32, 100), (16, 8, 264, W.BF16, 9), (1, 5, 8, W.BF16, 3),
    (3, 7, 100, W.F32, 30), (128, 1, 1024, W.BF16, 11), (4, 32, 16, W.BF16, 50), (8, 4, 520, W.F16, 25)])
def test_regroup_matches_oracle_and_inverts(T, oracle, P, E, d, dtype, mean_rows):
    rng = np.random.default_rng(P * 131 + E)
    cnt = rng.poisson(mean_rows, size=(P, E)).astype(np.int32)
    cnt[rng.integers(P), rng.integers(E)] = 0
    R = int(cnt.sum())
    cap = R + 17                                              # the buffers are larger than the data
    rows = W.to_storage(rng.standard_normal((cap, d)).astype(np.float32), dtype)
    ws = T.workspace(1, d, 1, 1, 1, dtype)
    x = to_dev(rows, dtype)
    out = torch.zeros_like(x)
    eoff = torch.empty((E + 1,), dtype=torch.int32, device="cuda")
    cnt_d = torch.from_numpy(cnt).cuda()
    T.tamoe_regroup(x, cnt_d, True, out, eoff, ws)
    torch.cuda.synchronize()
    ref, ref_off = oracle.regroup(np.ascontiguousarray(rows[:R]), dtype, cnt, True)
    got = to_host(out, dtype)
    np.testing.assert_array_equal(got[:R], ref)
    assert (got[R:] == 0).all()                               # rows beyond R are not touched
    np.testing.assert_array_equal(eoff.cpu().numpy(), ref_off)
    back = torch.zeros_like(x)
    T.tamoe_regroup(out, cnt_d, False, back, None, ws)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(to_host(back, dtype)[:R], rows[:R])


def test_regroup_clips_to_the_buffer_and_rejects_bad_shapes(T):
    cnt = torch.tensor([[5, 5], [5, 5]], dtype=torch.int32, device="cuda")      # 20 rows announced
    x = torch.arange(12 * 8, dtype=torch.float32, device="cuda").reshape(12, 8)   # room for 12
    out = torch.full_like(x, -1.0)
    ws = T.workspace(1, 8, 1, 1, 1, T.F32)
    T.tamoe_regroup(x, cnt, True, out, None, ws)
    torch.cuda.synchronize()
    o = out.cpu().numpy()
    # source-major rows 0..4 (s0e0) -> expert-major rows 0..4; rows 5..9 (s0e1) -> 10..14: only 10, 11 fit
    np.testing.assert_array_equal(o[:5], x.cpu().numpy()[:5])
    np.testing.assert_array_equal(o[10:12], x.cpu().numpy()[5:7])
    np.testing.assert_array_equal(o[5:7], x.cpu().numpy()[10:12])   # s1e0: the two rows of it that were received
    assert (o[7:10] == -1).all()                               # their sources lie beyond the buffer
    with pytest.raises(T.TamoeError):
        T.tamoe_regroup(x, torch.zeros((16, 16), dtype=torch.int32, device="cuda"), True, out, None, ws)


def test_regroup_at_the_benchmarked_size(T, oracle):
    """Large-shaped receive buffer (131072 rows of 8 KiB, P = 64 sources x E = 2 local experts), the
    launch configuration bench.py times; every row compared."""
    P, E, d, R = 64, 2, 4096, 131072
    rng = np.random.Generator(np.random.Philox(key=[4, 11]))
    share = rng.poisson(64, size=(P, E)).astype(np.float64) + 1.0
    cnt = np.floor(share / share.sum() * R).astype(np.int32)
    cnt[0, 0] += R - int(cnt.sum())
    rows = rng.integers(0, 1 << 16, size=(R, d), dtype=np.uint16)      # bit patterns: a pure permutation
    oracle.set_threads(oracle.max_threads())
    ref, ref_off = oracle.regroup(rows, W.BF16, cnt, True)
    x = torch.from_numpy(rows.view(np.int16)).cuda().view(torch.bfloat16)
    out = torch.empty_like(x)
    eoff = torch.empty((E + 1,), dtype=torch.int32, device="cuda")
    ws = T.workspace(1, d, 1, 1, 1, W.BF16)
    cnt_d = torch.from_numpy(cnt).cuda()
    T.tamoe_regroup(x, cnt_d, True, out, eoff, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_host(out, W.BF16), ref)
    np.testing.assert_array_equal(eoff.cpu().numpy(), ref_off)
    T.tamoe_regroup(out, cnt_d, False, x, None, ws)                      # and back, over the input
    torch.cuda.synchronize()
    assert np.array_equal(to_host(x, W.BF16), rows)
