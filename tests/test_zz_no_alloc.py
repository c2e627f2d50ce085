"""tamoe_dispatch_static (the dispatch for callers that cannot allocate: scratch inside the library's
device image) against tamoe_dispatch with a workspace: same bits, on two calls in a row, the second
on a smaller input, so that what the first call left in the shared scratch is in the way."""
import numpy as np
import pytest

import tamoe_workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def T():
    if not torch.cuda.is_available():
        pytest.fail("these tests need a GPU (run with -m 'not gpu' elsewhere)")
    import paper_2302_09915_amd as T

    T.lib()
    return T


def _outputs(S, d, N, P, k, dtype, dev):
    return {
        "send": torch.zeros((S * k, d), dtype=dtype, device=dev),
        "slot": torch.full((S, k), -7, dtype=torch.int32, device=dev),
        "kept": torch.full((N,), -7, dtype=torch.int32, device=dev),
        "off": torch.full((N + 1,), -7, dtype=torch.int32, device=dev),
        "scd": torch.full((P,), -7, dtype=torch.int32, device=dev),
    }


def _both(T, S, d, N, P, k, capv, skew, seed):
    dev = torch.device("cuda:0")
    idx = torch.from_numpy(W.random_routing(seed, S, N, k, skew)).to(dev)
    cap = np.full(N, capv, dtype=np.int32)
    cap[1::3] += 3
    cap = torch.from_numpy(cap).to(dev)
    x = torch.randn((S, d), device=dev, generator=torch.Generator(device=dev).manual_seed(seed)).to(torch.bfloat16)
    a = _outputs(S, d, N, P, k, x.dtype, dev)
    b = _outputs(S, d, N, P, k, x.dtype, dev)
    ws = T.workspace(S, d, N, P, k, T.BF16)
    T.tamoe_dispatch(x, idx, cap, N, P, a["send"], a["slot"], a["kept"], a["off"], a["scd"], ws)
    T.tamoe_dispatch_static(x, idx, cap, N, P, b["send"], b["slot"], b["kept"], b["off"], b["scd"])
    torch.cuda.synchronize()
    K = int(a["off"][-1].item())
    assert 0 < K <= S * k
    for name in ("slot", "kept", "off", "scd"):
        assert torch.equal(a[name], b[name]), name
    assert torch.equal(a["send"][:K].view(torch.int16), b["send"][:K].view(torch.int16))
    return K


def test_static_scratch_dispatch_matches_the_workspace_dispatch(T, oracle):
    K1 = _both(T, 20000, 256, 128, 64, 2, 400, 1.0, seed=21)      # 20 count tiles, drops
    K2 = _both(T, 3000, 64, 16, 4, 3, 600, 0.5, seed=22)          # smaller: 3 count tiles, other N and k
    assert K2 < K1
    # and against the oracle, so that the pair of equal results is also the right one
    S, N, P, k = 3000, 16, 4, 3
    idx = W.random_routing(22, S, N, k, 0.5)
    cap = np.full(N, 600, dtype=np.int32)
    cap[1::3] += 3
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    assert K == K2
    dev = torch.device("cuda:0")
    x = torch.zeros((S, 8), dtype=torch.bfloat16, device=dev)
    b = _outputs(S, 8, N, P, k, x.dtype, dev)
    T.tamoe_dispatch_static(x, torch.from_numpy(idx).to(dev), torch.from_numpy(cap).to(dev), N, P, b["send"],
                            b["slot"], b["kept"], b["off"], b["scd"])
    torch.cuda.synchronize()
    np.testing.assert_array_equal(b["slot"].cpu().numpy(), slot)
    np.testing.assert_array_equal(b["off"].cpu().numpy(), off)
    np.testing.assert_array_equal(b["scd"].cpu().numpy(), scd)


def test_static_scratch_dispatch_rejects_what_does_not_fit(T):
    dev = torch.device("cuda:0")
    S, d, N, P, k = 300 * 1024, 8, 128, 64, 8                    # 8 * 300 * 128 counters > 262144
    x = torch.zeros((S, d), dtype=torch.bfloat16, device=dev)
    idx = torch.zeros((S, k), dtype=torch.int32, device=dev)
    cap = torch.ones((N,), dtype=torch.int32, device=dev)
    b = _outputs(S, d, N, P, k, x.dtype, dev)
    with pytest.raises(T.TamoeError) as err:
        T.tamoe_dispatch_static(x, idx, cap, N, P, b["send"], b["slot"], b["kept"], b["off"], b["scd"])
    assert err.value.status == T.UNSUPPORTED and "built-in scratch" in err.value.message
    assert (b["slot"] == -7).all() and (b["kept"] == -7).all()     # nothing was enqueued
