"""The seeded input generators: reproducible bytes, the shapes of the five configurations, the
storage rounding, the two-tier topology table and the Zipf recipe."""
import numpy as np
import pytest

import tamoe_workloads as W


def test_configs_have_the_stated_shapes():
    spec = {"tiny": (512, 64, W.F32, 8, 1, 8), "small": (4096, 512, W.BF16, 16, 2, 16),
            "gpt_moe": (16384, 1024, W.BF16, 64, 2, 64), "skewed": (16384, 2048, W.BF16, 64, 1, 64),
            "large": (65536, 4096, W.BF16, 128, 2, 64)}
    for name, (S, d, dt, N, k, P) in spec.items():
        wl = W.WORKLOADS[name]
        assert (wl.S, wl.d, wl.dtype, wl.N, wl.k, wl.P) == (S, d, dt, N, k, P)
        assert wl.N % wl.P == 0 and wl.E == N // P
        assert (wl.d * wl.elem_bytes) % 16 == 0
    assert W.WORKLOADS["tiny"].seed == 0


def test_inputs_are_reproducible_and_have_the_stated_distribution():
    wl = W.WORKLOADS["small"]
    a, b = W.make_inputs(wl), W.make_inputs(wl)
    np.testing.assert_array_equal(a["x"], b["x"])
    np.testing.assert_array_equal(a["w"], b["w"])
    assert a["x"].dtype == np.uint16 and a["x"].shape == (wl.S, wl.d) and a["w"].shape == (wl.N, wl.d)
    x = W.storage_to_f64(a["x"], wl.dtype)
    w = W.storage_to_f64(a["w"], wl.dtype)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    assert abs(w.std() * np.sqrt(wl.d) - 1.0) < 0.05
    t = W.make_inputs(W.WORKLOADS["tiny"])
    assert t["x"].dtype == np.float32 and t["x"].shape == (512, 64)


def test_bf16_round_trip_and_ties():
    v = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 3.0e38, 1e-40], dtype=np.float32)
    bits = W.f32_to_bf16_bits(v)
    assert list(bits[:4]) == [0x3F80, 0x3F80, 0x3F82, 0xC020]          # ties to even
    back = W.bf16_bits_to_f32(bits)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(back), bits)      # idempotent
    assert np.abs(back[:4] - v[:4]).max() <= 2.0 ** -8


def test_two_tier_topology_table():
    beta, level = W.two_tier_topology(2, 4, 4.0)
    assert beta.shape == (8, 8) and level.dtype == np.int32
    assert (np.diag(beta) == 1.0).all() and (np.diag(level) == 0).all()
    assert beta[0, 3] == 1.0 and beta[0, 4] == 4.0 and beta[5, 2] == 4.0 and beta[6, 7] == 1.0
    np.testing.assert_array_equal(beta, beta.T)
    assert (level == (beta > 1.0)).all()


def test_zipf_recipe_gives_zipf_popularity_and_forces_drops():
    wl = W.WORKLOADS["skewed"]
    inp = W.make_inputs(wl, S=8192)
    x = W.storage_to_f64(inp["x"], wl.dtype)
    w = W.storage_to_f64(inp["w"], wl.dtype)
    assert (x[:, -1] == 1.0).all()                                     # the constant feature carrying the offsets
    share = np.bincount((x @ w.T).argmax(axis=1), minlength=wl.N) / 8192.0
    target = W.zipf_popularity(wl.N, wl.zipf_s)
    assert abs(share[0] - target[0]) < 0.03 and share[0] > 8 * share[20]
    assert np.abs(share[:8] - target[:8]).max() < 0.03
    # capacity factor 1.0: the most popular expert receives far more than S/N tokens
    assert share[0] * wl.N > 10


def test_random_routing_has_distinct_experts():
    idx = W.random_routing(3, 500, 16, 4, skew=1.0)
    assert idx.shape == (500, 4) and idx.dtype == np.int32
    assert all(len(set(r)) == 4 for r in idx) and idx.min() >= 0 and idx.max() < 16
    c = np.bincount(idx.ravel(), minlength=16)
    assert c[0] > c[15]


def test_paper_shapes_are_the_gpt_model_table():
    assert set(W.PAPER_SHAPES) == {"paper_switch_fp16", "paper_gshard_fp16", "paper_switch_fp32", "paper_gshard_fp32"}
    for name, wl in W.PAPER_SHAPES.items():
        assert wl.d == 1024 and wl.N == 64 and wl.P == 64 and wl.E == 1
        assert wl.k == (1 if "switch" in name else 2)
        assert wl.dtype == (W.F16 if "fp16" in name else W.F32)
        assert W.workload(name) is wl
    assert W.PAPER_SHAPES["paper_switch_fp16"].capacity_factor == 1.0
    assert W.PAPER_SHAPES["paper_gshard_fp16"].capacity_factor == 2.0
    assert W.workload("large") is W.WORKLOADS["large"]
    x = W.make_inputs(W.PAPER_SHAPES["paper_gshard_fp16"], S=64)["x"]
    assert x.dtype == np.uint16 and np.isfinite(W.storage_to_f64(x, W.F16)).all()
