"""Parity of the HIP path (through the C ABI) against the CPU oracle on a real MI355X.

Staging (same seeded inputs on both sides):
  A  scores: GPU fp32 logits vs oracle fp64 logits, normwise and elementwise, tol 1e-3 (bf16 and
     half-precision inputs) / 1e-5 (fp32 inputs);
  B  everything decided from the scores is compared with the oracle re-run on the GPU's own fp32
     scores: indices, counts, slots, kept, offsets, per-device rows bit-exact; weights, mean
     probabilities and the losses within 1e-5 relative;
  C  the send buffer is a bit copy;
  D  combine: against the oracle's fp64 sum of the same rows with the GPU's fp32 weights: within
     half an ulp of the storage type plus the fp32 accumulation error, and equal to the oracle's
     once-rounded output in all but a tiny fraction of elements (1-ulp flips at rounding ties);
  E  end to end: the loss from the oracle's own scores vs the GPU's, 1e-3 (2-byte storage) / 1e-5 (fp32).
"""
import math

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

    T.lib()          # raises if the HIP library is missing: there is no fallback
    return T


# ---------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------
def to_dev(a: np.ndarray, dtype: int):
    t = torch.from_numpy(a)
    if dtype == W.BF16:
        t = t.view(torch.int16).view(torch.bfloat16)
    elif dtype == W.F16:
        t = t.view(torch.int16).view(torch.float16)
    return t.cuda()


def to_host(t, dtype: int) -> np.ndarray:
    if dtype in (W.BF16, W.F16):
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def torch_dtype(dtype: int):
    return {W.F32: torch.float32, W.BF16: torch.bfloat16, W.F16: torch.float16}[dtype]


def ulp_of(v: np.ndarray, dtype: int) -> np.ndarray:
    """Spacing of the storage type at |v| (float64 in, float64 out); below the smallest normal value
    the spacing is that of the subnormals."""
    mant, e_min = {W.F32: (23, -126), W.BF16: (7, -126), W.F16: (10, -14)}[dtype]
    a = np.abs(v)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** e_min)))
    return 2.0 ** (e - mant)


def flip_bound(dtype: int, k: int) -> float:
    """Share of elements that may differ by one storage ulp from the oracle's once-rounded value: the
    fp32 accumulation error (about (k+1) roundings of 2^-24) lets a sum cross a rounding boundary of
    the storage type with probability ~ 2 * error / ulp; bfloat16: ulp 2^-8 relative, half: 2^-11."""
    return 1e-3 if dtype == W.BF16 else max(1e-3, 4.0 * (k + 1) * 2.0 ** -24 / 2.0 ** -11)


def check_logits(gpu: np.ndarray, ref: np.ndarray, dtype: int):
    tol = 1e-3 if dtype != W.F32 else 1e-5
    diff = np.abs(gpu.astype(np.float64) - ref)
    assert diff.max() <= tol * np.abs(ref).max()
    rms = math.sqrt(float((ref ** 2).mean()))
    assert (diff <= tol * (np.abs(ref) + rms)).all()


def check_routing(T, oracle, g, ref, N, k):
    """g: GPU outputs (numpy), ref: oracle.route_from_logits on the GPU's scores."""
    np.testing.assert_array_equal(g["topk_idx"], ref["topk_idx"])
    np.testing.assert_array_equal(g["c_expert"], ref["c_expert"])
    np.testing.assert_array_equal(g["c_device"], ref["c_device"])
    np.testing.assert_allclose(g["topk_w"], ref["topk_w"], rtol=1e-5, atol=1e-30)
    np.testing.assert_allclose(g["m"], ref["m"], rtol=1e-5, atol=1e-12)
    np.testing.assert_array_equal(g["slot"], ref["slot"])
    np.testing.assert_array_equal(g["kept_expert"], ref["kept"])
    np.testing.assert_array_equal(g["expert_offset"], ref["off"])
    np.testing.assert_array_equal(g["send_count_dev"], ref["send_count_dev"])
    assert g["l_topo"] == pytest.approx(ref["l_topo"], rel=1e-5)
    assert g["l_aux"] == pytest.approx(ref["l_aux"], rel=1e-5)
    assert g["c_expert"].sum() == g["topk_idx"].size


def check_combine(y_gpu: np.ndarray, y_exact: np.ndarray, y_ref: np.ndarray, mag: np.ndarray, dtype: int, k: int):
    """mag = sum_j |w_j * recv_j| elementwise (bounds the fp32 accumulation error)."""
    yv = W.storage_to_f64(y_gpu, dtype)
    arith = 4.0 * k * 2.0 ** -24 * mag
    bound = 0.5 * ulp_of(y_exact, dtype) + arith + 2.0 ** -149
    assert (np.abs(yv - y_exact) <= bound).all()
    if dtype != W.F32:
        # the storage ulp dwarfs the fp32 accumulation error: the once-rounded results agree except
        # where the exact sum sits on a rounding boundary
        flips = (y_gpu != y_ref)
        flips &= ~((W.storage_to_f64(y_ref, dtype) == 0) & (yv == 0))      # +0 / -0 are the same value
        assert flips.mean() <= flip_bound(dtype, k)
    else:
        assert (np.abs(yv - y_exact) <= 1e-5 * np.maximum(np.abs(y_exact), mag)).all()


def gpu_path(T, wl_like, x_np, w_np, penalty, cap, want_logits=True, fused=False):
    """Runs gate -> losses -> dispatch -> combine (identity expert) through the C ABI: the separate
    entry points, or (fused) tamoe_gate_dispatch for everything up to the send buffer."""
    dt = wl_like["dtype"]
    N, P, k = wl_like["N"], wl_like["P"], wl_like["k"]
    x = to_dev(x_np, dt)
    w = to_dev(w_np, dt)
    S, d = x.shape
    ws = T.workspace(S, d, N, P, k, dt)
    pen = torch.from_numpy(penalty.astype(np.float32)).cuda()
    capd = torch.from_numpy(cap.astype(np.int32)).cuda()
    if fused:
        g = dsp = T.gate_dispatch(x, w, P, k, pen, capd, want_logits=want_logits, ws=ws)
        l_topo = g["loss"] if S > 0 else None
    else:
        g = T.gate(x, w, P, k, want_logits=want_logits, ws=ws)
        l_topo = T.aux_loss(g["m"], g["c_expert"], pen, P, S) if S > 0 else None
        dsp = T.dispatch(x, g["topk_idx"], capd, N, P, ws=ws)
    l_aux = T.aux_loss(g["m"], g["c_expert"], None, P, S) if S > 0 else None
    torch.cuda.synchronize()
    K = int(dsp["expert_offset"][-1].item())
    y = T.combine(dsp["send"], K, dsp["slot"], g["topk_w"], d=d)
    torch.cuda.synchronize()
    out = {
        "logits": g["logits"].cpu().numpy() if want_logits else None,
        "topk_idx": g["topk_idx"].cpu().numpy(), "topk_w": g["topk_w"].cpu().numpy(),
        "m": g["m"].cpu().numpy(), "c_expert": g["c_expert"].cpu().numpy(), "c_device": g["c_device"].cpu().numpy(),
        "l_topo": float(l_topo.item()) if l_topo is not None else None,
        "l_aux": float(l_aux.item()) if l_aux is not None else None,
        "slot": dsp["slot"].cpu().numpy(), "kept_expert": dsp["kept_expert"].cpu().numpy(),
        "expert_offset": dsp["expert_offset"].cpu().numpy(), "send_count_dev": dsp["send_count_dev"].cpu().numpy(),
        "K": K, "send_t": dsp["send"], "y": to_host(y, dt),
    }
    return out


def full_parity(T, oracle, spec, x_np, w_np, penalty, cap, sample=None):
    """All stages.  `sample` = token indices for the stages that are too slow on the CPU at full
    size (scores, combine); None = every token."""
    dt, N, P, k = spec["dtype"], spec["N"], spec["P"], spec["k"]
    S, d = x_np.shape
    g = gpu_path(T, spec, x_np, w_np, penalty, cap)
    rows = np.arange(S) if sample is None else np.asarray(sample)

    # A: scores
    ref_lg = oracle.logits(np.ascontiguousarray(x_np[rows]), w_np, dt)
    check_logits(g["logits"][rows], ref_lg, dt)

    # B: routing from the GPU's own scores (cheap: every token)
    ref = oracle.route_from_logits(g["logits"].astype(np.float64), k, P, penalty, cap)
    check_routing(T, oracle, g, ref, N, k)
    assert g["K"] == ref["K"]

    # C: send buffer (every row)
    send = to_host(g["send_t"][: g["K"]], dt)
    ref_send = oracle.scatter(x_np, dt, ref["slot"], ref["K"])
    np.testing.assert_array_equal(send, ref_send)

    # D: combine on the sampled tokens, identity expert, GPU weights; in blocks of tokens so that the
    # fp64 copies of a full-size batch stay small
    block = max(1, (1 << 25) // max(d, 1))
    for r0 in range(0, len(rows), block):
        rb = rows[r0:r0 + block]
        slot_s = ref["slot"][rb]
        used = np.unique(slot_s[slot_s >= 0])
        remap = -np.ones(max(ref["K"], 1), dtype=np.int32)
        remap[used] = np.arange(len(used), dtype=np.int32)
        slot_sub = np.where(slot_s >= 0, remap[np.maximum(slot_s, 0)], -1).astype(np.int32)
        recv_sub = np.ascontiguousarray(ref_send[used]) if len(used) else np.zeros((1, d), dtype=ref_send.dtype)
        wg = g["topk_w"][rb].astype(np.float64)
        y_exact, y_ref = oracle.combine(recv_sub, dt, slot_sub, wg)
        xv = np.abs(W.storage_to_f64(np.ascontiguousarray(x_np[rb]), dt))
        mag = (np.where(slot_s >= 0, np.abs(wg), 0.0).sum(axis=1))[:, None] * xv
        check_combine(g["y"][rb], y_exact, y_ref, mag, dt, k)

    # E: end to end, oracle on its own scores (needs all tokens' scores: only when not sampled)
    if sample is None and S > 0:
        own = oracle.route_from_logits(ref_lg, k, P, penalty, cap)
        tol = 1e-3 if dt != W.F32 else 1e-5
        assert g["l_topo"] == pytest.approx(own["l_topo"], rel=tol)
        assert g["l_aux"] == pytest.approx(own["l_aux"], rel=tol)

    # The fused entry point (gate, loss and dispatch in three launches): what is decided from the scores
    # must be the bits of the separate calls, which were just checked against the oracle; the two sums
    # that it folds in another fixed order (m, the loss) are compared with the oracle directly.
    f = gpu_path(T, spec, x_np, w_np, penalty, cap, fused=True)
    for key in ("logits", "topk_idx", "topk_w", "c_expert", "c_device", "slot", "kept_expert", "expert_offset",
                "send_count_dev", "y"):
        np.testing.assert_array_equal(f[key], g[key], err_msg=f"fused {key}")
    assert f["K"] == g["K"]
    assert torch.equal(f["send_t"][: f["K"]].view(torch.uint8), g["send_t"][: g["K"]].view(torch.uint8))
    np.testing.assert_allclose(f["m"], ref["m"], rtol=1e-5, atol=1e-12)
    if S > 0:
        assert f["l_topo"] == pytest.approx(ref["l_topo"], rel=1e-5)
        assert f["l_aux"] == pytest.approx(ref["l_aux"], rel=1e-5)
    return g, ref


def spec_of(wl):
    return {"dtype": wl.dtype, "N": wl.N, "P": wl.P, "k": wl.k}


# ---------------------------------------------------------------------------
# the five configurations, both capacity modes
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny", "small", "gpt_moe", "skewed"])
@pytest.mark.parametrize("cap_mode", [0, 1])
def test_config_parity(T, oracle, name, cap_mode):
    wl = W.WORKLOADS[name]
    oracle.set_threads(oracle.max_threads())
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    rank = 0 if cap_mode == 0 else wl.P // 2 + 1
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, rank, wl.k, wl.S, wl.capacity_factor, cap_mode)
    g, ref = full_parity(T, oracle, spec_of(wl), inp["x"], inp["w"], pen.astype(np.float64), cap)
    if name == "skewed":
        assert ref["K"] < wl.k * wl.S * 0.6, "the skewed configuration must drop a large share of the pairs"
        share = ref["c_expert"] / ref["c_expert"].sum()
        assert share[0] > 0.2 and share[0] > 5 * share[16]


@pytest.mark.parametrize("name", ["small", "gpt_moe", "skewed"])
def test_config_parity_half_precision(T, oracle, name):
    """The same configurations with half-precision storage, the data type of the paper's own runs on its
    first cluster (GPT model table); inputs drawn as for bf16 and rounded to half precision."""
    import dataclasses

    wl = dataclasses.replace(W.WORKLOADS[name], dtype=W.F16)
    oracle.set_threads(oracle.max_threads())
    inp = W.make_inputs(wl)
    assert inp["x"].dtype == np.uint16
    beta, level = W.topology(wl)
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    g, ref = full_parity(T, oracle, spec_of(wl), inp["x"], inp["w"], pen.astype(np.float64), cap)


@pytest.mark.parametrize("name", sorted(W.PAPER_SHAPES))
def test_paper_shapes_parity(T, oracle, name):
    """The shapes of the paper's own runs (GPT model table): both gates, FP16 and FP32 storage."""
    wl = W.PAPER_SHAPES[name]
    oracle.set_threads(oracle.max_threads())
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, wl.P // 2 + 1, wl.k, wl.S, wl.capacity_factor, 0)
    full_parity(T, oracle, spec_of(wl), inp["x"], inp["w"], pen.astype(np.float64), cap)


ROUTED_KEYS = ("topk_idx", "topk_w", "m", "c_expert", "c_device", "slot", "kept_expert", "expert_offset",
               "send_count_dev", "y")


@pytest.mark.parametrize("cap_mode", [0, 1])
def test_large_config_parity(T, oracle, cap_mode):
    """Full size, the launch configuration the benchmark times: every stage on every token, under the
    uniform capacity (rank 0) and under the capacity proportional to the target pattern (an interior
    rank; a random gate then loses a large share of its pairs).  The benchmark calls the gate without
    the optional scores output: that call must give the same bits as the one checked here."""
    wl = W.WORKLOADS["large"]
    oracle.set_threads(oracle.max_threads())
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    rank = 0 if cap_mode == 0 else wl.P // 2 + 1
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, rank, wl.k, wl.S, wl.capacity_factor, cap_mode)
    g, ref = full_parity(T, oracle, spec_of(wl), inp["x"], inp["w"], pen.astype(np.float64), cap)
    if cap_mode == 1:
        assert ref["K"] < 0.75 * wl.k * wl.S, "the proportional capacity must drop pairs of a random gate"
        assert (ref["slot"] < 0).all(axis=1).any(), "some token must lose every choice"
    send_a = g.pop("send_t")[: g["K"]].view(torch.int16).cpu()
    b = gpu_path(T, spec_of(wl), inp["x"], inp["w"], pen, cap, want_logits=False)
    for key in ROUTED_KEYS:
        np.testing.assert_array_equal(g[key], b[key], err_msg=key)
    assert g["l_topo"] == b["l_topo"] and g["l_aux"] == b["l_aux"] and g["K"] == b["K"]
    assert torch.equal(send_a, b["send_t"][: b["K"]].view(torch.int16).cpu())


# Shapes that reach the gate's eight-wavefront workgroups (more than 32 experts and at least 65 281
# tokens) in every instantiation: three storage types x (up to 64 | up to 128 experts) x (hidden size
# a multiple of the 128-byte K chunk | with a K tail).  Small hidden sizes keep the oracle cheap.
@pytest.mark.parametrize("dtype,d,N,P,k", [
    (W.BF16, 128, 64, 64, 1), (W.BF16, 200, 48, 16, 2), (W.BF16, 192, 128, 64, 2), (W.BF16, 72, 96, 8, 3),
    (W.F16, 64, 64, 8, 2), (W.F16, 88, 40, 10, 1), (W.F16, 128, 128, 64, 2), (W.F16, 264, 96, 32, 2),
    (W.F32, 96, 64, 64, 2), (W.F32, 100, 33, 11, 1), (W.F32, 64, 128, 64, 2), (W.F32, 36, 96, 96, 4),
])
def test_eight_wavefront_gate_shapes(T, oracle, dtype, d, N, P, k):
    S = 66000                                   # 258 workgroups of 256 tokens, the last one ragged
    oracle.set_threads(oracle.max_threads())
    rng = np.random.default_rng(7 * d + N)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    w = W.to_storage((rng.standard_normal((N, d)) / math.sqrt(d)).astype(np.float32), dtype)
    beta = rng.uniform(1.0, 9.0, size=(P, P))
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, None, P, N, P // 3, k, S, 1.1, (d // 8) % 2)
    full_parity(T, oracle, {"dtype": dtype, "N": N, "P": P, "k": k}, x, w, pen.astype(np.float64), cap)


# ---------------------------------------------------------------------------
# ragged shapes, small and odd sizes, limits
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,S,d,N,P,k,cf", [
    (W.BF16, 1, 8, 1, 1, 1, 1.0),          # smallest everything
    (W.BF16, 33, 72, 5, 5, 2, 1.0),        # ragged tile, K tail, odd N
    (W.BF16, 129, 200, 48, 16, 3, 0.5),    # N not a multiple of 32, E = 3
    (W.BF16, 1000, 64, 128, 64, 8, 1.0),   # k at the limit, N at the limit
    (W.BF16, 2500, 264, 96, 8, 2, 2.0),    # several count tiles, ragged end
    (W.BF16, 70000, 16, 32, 4, 1, 1.1),    # many tokens, tiny rows
    (W.BF16, 70001, 1024, 96, 8, 3, 0.9),  # 410 MiB of rows to send: the fused call's scatter writes them with streaming stores
    (W.BF16, 60000, 1000, 64, 8, 2, 1.0),  # the same with rows that are no multiple of 1 KiB (a wavefront spans tokens)
    (W.F16, 70001, 1000, 40, 8, 1, 1.5),   # and with one choice (two chunks per thread)
    (W.F16, 33, 72, 5, 5, 2, 1.0),         # half precision: ragged tile, K tail, odd N
    (W.F16, 2500, 264, 96, 8, 2, 2.0),
    (W.F16, 1000, 64, 128, 64, 8, 1.0),
    (W.F16, 40000, 128, 64, 8, 1, 1.0),    # four-wavefront workgroups
    (W.F32, 1, 4, 2, 1, 2, 1.0),
    (W.F32, 77, 36, 33, 11, 4, 0.7),
    (W.F32, 1500, 100, 128, 2, 2, 1.0),
    (W.F32, 300, 1024, 64, 64, 1, 1.0),
])
def test_odd_shapes(T, oracle, dtype, S, d, N, P, k, cf):
    oracle.set_threads(oracle.max_threads())
    rng = np.random.default_rng(S * 31 + d)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    w = W.to_storage((rng.standard_normal((N, d)) / math.sqrt(d)).astype(np.float32), dtype)
    beta = rng.uniform(1.0, 9.0, size=(P, P))
    rank = P // 2
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, None, P, N, rank, k, S, cf, 1)
    full_parity(T, oracle, {"dtype": dtype, "N": N, "P": P, "k": k}, x, w, pen.astype(np.float64), cap)


def _random_shape(i):
    """Seeded random shape inside the library's limits: ragged S, d any multiple of 16 bytes, any N % P == 0."""
    rng = np.random.default_rng(1000 + i)
    dtype = (W.F32, W.BF16, W.F16, W.BF16)[i % 4]
    P = int(rng.choice([1, 2, 3, 4, 6, 8, 16, 32, 64]))
    E = int(rng.integers(1, max(2, 128 // P + 1)))
    N = P * E
    k = int(rng.integers(1, min(N, 8) + 1))
    S = int(rng.choice([rng.integers(1, 300), rng.integers(300, 5000), rng.integers(5000, 40000)]))
    unit = 4 if dtype == W.F32 else 8
    d = unit * int(rng.choice([rng.integers(1, 9), rng.integers(9, 80), rng.integers(80, 300)]))
    if S * d > 6_000_000:                                   # keep the oracle's fp64 score product to seconds
        S = max(1, 6_000_000 // d)
    cf = float(rng.choice([0.5, 1.0, 1.25, 2.0]))
    return dtype, S, d, N, P, k, cf


@pytest.mark.parametrize("i", range(40))
def test_random_shapes(T, oracle, i):
    dtype, S, d, N, P, k, cf = _random_shape(i)
    print(f"shape {i}: dtype={dtype} S={S} d={d} N={N} P={P} k={k} cf={cf}", flush=True)
    oracle.set_threads(oracle.max_threads())
    rng = np.random.default_rng(2000 + i)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), dtype)
    w = W.to_storage((rng.standard_normal((N, d)) / math.sqrt(d)).astype(np.float32), dtype)
    beta = rng.uniform(1.0, 9.0, size=(P, P))
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, None, P, N, int(rng.integers(P)), k, S, cf, i % 2)
    full_parity(T, oracle, {"dtype": dtype, "N": N, "P": P, "k": k}, x, w, pen.astype(np.float64), cap)


def test_empty_input(T):
    N, P, k, d = 8, 4, 2, 64
    x = torch.empty((0, d), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros((N, d), dtype=torch.bfloat16, device="cuda")
    g = T.gate(x, w, P, k)
    cap = torch.full((N,), 5, dtype=torch.int32, device="cuda")
    dsp = T.dispatch(x, g["topk_idx"], cap, N, P)
    y = T.combine(dsp["send"], 0, dsp["slot"], g["topk_w"], d=d)
    torch.cuda.synchronize()
    assert g["c_expert"].sum().item() == 0 and g["c_device"].sum().item() == 0
    assert (g["m"] == 0).all()
    assert dsp["kept_expert"].sum().item() == 0 and (dsp["expert_offset"] == 0).all()
    assert dsp["send_count_dev"].sum().item() == 0 and y.shape == (0, d)
    pen = torch.full((N,), 1.0 / N, device="cuda")
    f = T.gate_dispatch(x, w, P, k, pen, cap)
    torch.cuda.synchronize()
    assert f["c_expert"].sum().item() == 0 and (f["m"] == 0).all() and f["loss"].item() == 0.0
    assert f["kept_expert"].sum().item() == 0 and (f["expert_offset"] == 0).all()
    assert f["send_count_dev"].sum().item() == 0 and f["c_device"].sum().item() == 0


@pytest.mark.parametrize("capv", [0, 1, 45, 10 ** 6])
def test_fused_call_options(T, oracle, capv):
    """tamoe_gate_dispatch without a penalty (the loss is then l_aux of Section 3.1), without a loss
    pointer, and under capacities that keep nothing, one row, some rows, everything."""
    S, d, N, P, k = 3001, 192, 48, 8, 2
    rng = np.random.default_rng(capv + 3)
    x_np = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), W.BF16)
    w_np = W.to_storage((rng.standard_normal((N, d)) / np.sqrt(d)).astype(np.float32), W.BF16)
    cap = np.full(N, capv, dtype=np.int32)
    if capv == 45:
        cap[::5] = 0
        cap[1::7] = 10 ** 6
    x, w = to_dev(x_np, W.BF16), to_dev(w_np, W.BF16)
    capd = torch.from_numpy(cap).cuda()
    f = T.gate_dispatch(x, w, P, k, None, capd)
    torch.cuda.synchronize()
    ref = oracle.route_from_logits(f["logits"].cpu().numpy().astype(np.float64), k, P, np.full(N, 1.0 / N), cap)
    assert f["loss"].item() == pytest.approx(ref["l_aux"], rel=1e-5)
    np.testing.assert_array_equal(f["topk_idx"].cpu().numpy(), ref["topk_idx"])
    np.testing.assert_array_equal(f["slot"].cpu().numpy(), ref["slot"])
    np.testing.assert_array_equal(f["kept_expert"].cpu().numpy(), ref["kept"])
    np.testing.assert_array_equal(f["expert_offset"].cpu().numpy(), ref["off"])
    np.testing.assert_array_equal(f["send_count_dev"].cpu().numpy(), ref["send_count_dev"])
    K = ref["K"]
    assert K == {0: 0, 1: N, 10 ** 6: S * k}.get(capv, K)
    np.testing.assert_array_equal(to_host(f["send"][:K], W.BF16), oracle.scatter(x_np, W.BF16, ref["slot"], K))
    # no loss pointer: everything else as before
    g = T.gate_dispatch(x, w, P, k, None, capd)
    g["loss"].fill_(-7.0)
    T.tamoe_gate_dispatch(x, w, P, k, None, capd, g["logits"], g["topk_idx"], g["topk_w"], g["m"], g["c_expert"],
                          g["c_device"], None, g["send"], g["slot"], g["kept_expert"], g["expert_offset"],
                          g["send_count_dev"], T.workspace(S, d, N, P, k, W.BF16))
    torch.cuda.synchronize()
    assert g["loss"].item() == -7.0
    for key in ("topk_idx", "topk_w", "m", "c_expert", "c_device", "slot", "kept_expert", "expert_offset",
                "send_count_dev"):
        assert torch.equal(f[key], g[key]), key
    assert torch.equal(f["send"][:K].view(torch.int16), g["send"][:K].view(torch.int16))


# ---------------------------------------------------------------------------
# selection stage fed given scores: ties, extreme values
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("S,N,P,k,ties", [(1000, 16, 4, 3, True), (777, 64, 8, 2, True), (513, 128, 1, 8, True),
                                          (4000, 8, 8, 1, False), (100, 40, 10, 5, False)])
def test_select_on_given_scores(T, oracle, S, N, P, k, ties):
    lg = W.random_logits(S + N, S, N, ties=ties)
    if not ties:
        lg = lg * np.float32(20.0)            # wide dynamic range: exp underflows for most experts
    out = T.select(torch.from_numpy(lg).cuda(), P, k)
    torch.cuda.synchronize()
    pen = np.full(N, 1.0 / N)
    ref = oracle.route_from_logits(lg.astype(np.float64), k, P, pen, np.full(N, S * k, dtype=np.int32))
    np.testing.assert_array_equal(out["topk_idx"].cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(out["topk_w"].cpu().numpy(), ref["topk_w"], rtol=1e-5, atol=1e-37)
    np.testing.assert_allclose(out["m"].cpu().numpy(), ref["m"], rtol=1e-5, atol=1e-12)
    np.testing.assert_array_equal(out["c_expert"].cpu().numpy(), ref["c_expert"])
    np.testing.assert_array_equal(out["c_device"].cpu().numpy(), ref["c_device"])


def test_all_equal_scores_pick_the_first_k(T):
    lg = torch.zeros((70, 12), dtype=torch.float32, device="cuda")
    out = T.select(lg, 3, 4)
    torch.cuda.synchronize()
    assert (out["topk_idx"].cpu() == torch.arange(4, dtype=torch.int32)[None, :]).all()
    np.testing.assert_allclose(out["topk_w"].cpu().numpy(), 1.0 / 12, rtol=1e-6)


# ---------------------------------------------------------------------------
# dispatch fed given routing: capacities, skew, bad indices; combine on foreign rows
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("S,N,P,k,capv,skew", [
    (5000, 16, 4, 2, 300, 1.5), (3000, 64, 64, 1, 0, 0.0), (2049, 128, 64, 4, 10 ** 6, 0.5),
    (100, 8, 2, 8, 37, 0.0), (1025, 4, 4, 2, 1, 3.0)])
def test_dispatch_on_given_routing(T, oracle, S, N, P, k, capv, skew):
    d = 32
    idx = W.random_routing(S + k, S, N, k, skew)
    cap = np.full(N, capv, dtype=np.int32)
    if capv > 0:
        cap[1::3] += 5
    rng = np.random.default_rng(1)
    x = W.to_storage(rng.standard_normal((S, d)).astype(np.float32), W.BF16)
    dsp = T.dispatch(to_dev(x, W.BF16), torch.from_numpy(idx).cuda(), torch.from_numpy(cap).cuda(), N, P)
    torch.cuda.synchronize()
    slot, kept, off, scd, K = oracle.slots(idx, cap, P)
    np.testing.assert_array_equal(dsp["slot"].cpu().numpy(), slot)
    np.testing.assert_array_equal(dsp["kept_expert"].cpu().numpy(), kept)
    np.testing.assert_array_equal(dsp["expert_offset"].cpu().numpy(), off)
    np.testing.assert_array_equal(dsp["send_count_dev"].cpu().numpy(), scd)
    np.testing.assert_array_equal(to_host(dsp["send"][:K], W.BF16), oracle.scatter(x, W.BF16, slot, K))


def test_dispatch_treats_out_of_range_experts_as_dropped(T, oracle):
    S, N, P, k, d = 600, 8, 4, 2, 16
    idx = W.random_routing(5, S, N, k)
    bad = idx.copy()
    bad[::7, 1] = N + 3
    bad[3::11, 0] = -2
    cap = np.full(N, 50, dtype=np.int32)
    x = np.arange(S * d, dtype=np.float32).reshape(S, d)
    dsp = T.dispatch(torch.from_numpy(x).cuda(), torch.from_numpy(bad).cuda(), torch.from_numpy(cap).cuda(), N, P)
    torch.cuda.synchronize()
    slot = dsp["slot"].cpu().numpy()
    invalid = (bad < 0) | (bad >= N)
    assert (slot[invalid] == -1).all()
    # the valid pairs are ranked as if the bad ones were absent: oracle on a routing where the bad
    # pairs point at an extra expert with zero capacity
    patched = np.where(invalid, N, bad).astype(np.int32)
    oslot, okept, ooff, _, K = oracle.slots(patched, np.concatenate([cap, [0]]).astype(np.int32), 1)
    np.testing.assert_array_equal(slot, oslot)
    np.testing.assert_array_equal(dsp["kept_expert"].cpu().numpy(), okept[:N])
    np.testing.assert_array_equal(to_host(dsp["send"][:K], W.F32), oracle.scatter(x, W.F32, oslot, K))


@pytest.mark.parametrize("dtype,k", [(W.BF16, 2), (W.BF16, 1), (W.F32, 3), (W.BF16, 5)])
def test_combine_on_foreign_rows(T, oracle, dtype, k):
    """recv is not the send buffer: catches a combine that reads x or the wrong row."""
    S, d, K = 3000, 136, 4500
    rng = np.random.default_rng(k)
    recv = W.to_storage(rng.standard_normal((K, d)).astype(np.float32), dtype)
    slot = rng.integers(-1, K, size=(S, k)).astype(np.int32)
    slot[5] = -1
    slot[6, 0] = K + 10            # beyond K_rows: ignored like a dropped pair
    wgt = rng.uniform(0.0, 1.0, size=(S, k)).astype(np.float32)
    y = T.combine(to_dev(recv, dtype), K, torch.from_numpy(slot).cuda(), torch.from_numpy(wgt).cuda())
    torch.cuda.synchronize()
    oslot = np.where(slot >= K, -1, slot).astype(np.int32)
    y_exact, y_ref = oracle.combine(recv, dtype, oslot, wgt.astype(np.float64))
    rv = np.abs(W.storage_to_f64(recv, dtype))
    mag = np.zeros((S, d))
    for j in range(k):
        ok = oslot[:, j] >= 0
        mag[ok] += wgt[ok, j:j + 1].astype(np.float64) * rv[oslot[ok, j]]
    check_combine(to_host(y, dtype), y_exact, y_ref, mag, dtype, k)
    assert (W.storage_to_f64(to_host(y, dtype), dtype)[5] == 0).all()


# ---------------------------------------------------------------------------
# determinism, optional outputs, losses
# ---------------------------------------------------------------------------
def test_runs_are_bitwise_repeatable_and_logits_are_optional(T):
    wl = W.WORKLOADS["small"]
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    _, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    a = gpu_path(T, spec_of(wl), inp["x"], inp["w"], pen, cap, want_logits=True)
    b = gpu_path(T, spec_of(wl), inp["x"], inp["w"], pen, cap, want_logits=False)
    for key in ROUTED_KEYS:
        np.testing.assert_array_equal(a[key], b[key], err_msg=key)
    assert a["l_topo"] == b["l_topo"] and a["K"] == b["K"]
    assert torch.equal(a["send_t"][: a["K"]].view(torch.int16), b["send_t"][: b["K"]].view(torch.int16))


def test_bound_calls_repeat_the_call_they_were_made_from(T):
    """T.bind: arguments marshalled once, same launches, same bits."""
    wl = W.WORKLOADS["small"]
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    _, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    x, w = to_dev(inp["x"], wl.dtype), to_dev(inp["w"], wl.dtype)
    pen_d, cap_d = torch.from_numpy(pen).cuda(), torch.from_numpy(cap).cuda()
    a = T.gate_dispatch(x, w, wl.P, wl.k, pen_d, cap_d, want_logits=False)
    ya = T.combine(a["send"], wl.S * wl.k, a["slot"], a["topk_w"])
    b = {key: (torch.zeros_like(v) if v is not None else None) for key, v in a.items()}
    yb = torch.zeros_like(ya)
    ws = T.workspace(wl.S, wl.d, wl.N, wl.P, wl.k, wl.dtype)
    calls = [T.bind(T.tamoe_gate_dispatch, x, w, wl.P, wl.k, pen_d, cap_d, None, b["topk_idx"], b["topk_w"], b["m"],
                    b["c_expert"], b["c_device"], b["loss"], b["send"], b["slot"], b["kept_expert"],
                    b["expert_offset"], b["send_count_dev"], ws),
             T.bind(T.tamoe_combine, b["send"], wl.S * wl.k, b["slot"], b["topk_w"], yb)]
    for _ in range(2):
        for c in calls:
            c()
    torch.cuda.synchronize()
    K = int(a["expert_offset"][-1].item())
    for key in ("topk_idx", "topk_w", "m", "c_expert", "c_device", "loss", "slot", "kept_expert", "expert_offset",
                "send_count_dev"):
        assert torch.equal(a[key], b[key]), key
    assert torch.equal(a["send"][:K].view(torch.int16), b["send"][:K].view(torch.int16))
    assert torch.equal(ya.view(torch.int16), yb.view(torch.int16))


def test_aux_loss_closed_forms_on_device(T):
    """Uniform routing: l_topo = k/E for any penalty that sums to one; l_aux = k/N."""
    N, P, k, S = 64, 32, 2, 4096
    m = torch.full((N,), 1.0 / N, device="cuda")
    c = torch.full((N,), k * S // N, dtype=torch.int32, device="cuda")
    beta, level = W.two_tier_topology(4, 8, 6.0)
    _, pen, _ = T.tamoe_topo_pattern(beta, level, P, N, 5, k, S, 1.0, 0)
    lt = T.aux_loss(m, c, torch.from_numpy(pen).cuda(), P, S).item()
    la = T.aux_loss(m, c, None, P, S).item()
    assert lt == pytest.approx(k / (N // P), rel=1e-5)
    assert la == pytest.approx(k / N, rel=1e-5)


# ---------------------------------------------------------------------------
# measurement aids: the library's kernel trace, the benchmark's yardstick kernels
# ---------------------------------------------------------------------------
def test_kernel_trace_brackets_launches(T):
    w_in = torch.rand((4096, 2), device="cuda") + 0.1
    out = torch.empty_like(w_in)
    T.tamoe_trace_start(8)
    for _ in range(3):
        T.tamoe_renorm_topk(w_in, out)
    n = T.tamoe_trace_stop()
    assert n == 3
    for i in range(n):
        name, ms = T.tamoe_trace_get(i)
        assert name == "renorm_topk_kernel" and 0.0 < ms < 50.0
    # a filter on another kernel's name records nothing; clearing it records again
    T.tamoe_trace_filter("combine_kernel")
    T.tamoe_trace_start(8)
    T.tamoe_renorm_topk(w_in, out)
    assert T.tamoe_trace_stop() == 0
    T.tamoe_trace_filter(None)
    T.tamoe_trace_start(1)
    T.tamoe_renorm_topk(w_in, out)
    T.tamoe_renorm_topk(w_in, out)            # beyond the capacity: not recorded, still executed
    assert T.tamoe_trace_stop() == 1
    T.tamoe_trace_clear()
    with pytest.raises(T.TamoeError):
        T.tamoe_trace_get(0)


def test_bench_copy_probe_copies():
    from paper_2302_09915_amd import bench_aids as B

    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    B.copy_probe(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


@pytest.mark.parametrize("fused", [False, True])
def test_step_can_be_captured_in_a_graph(T, oracle, fused):
    """The library only enqueues kernels on the given stream (no allocation, no memset), so a whole
    step replays from a HIP graph; every replay must reproduce the eager result."""
    wl = W.WORKLOADS["small"]
    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    _, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, 0, wl.k, wl.S, wl.capacity_factor, 0)
    x, w = to_dev(inp["x"], wl.dtype), to_dev(inp["w"], wl.dtype)
    S, d, N, P, k = wl.S, wl.d, wl.N, wl.P, wl.k
    dev = x.device
    ws = T.workspace(S, d, N, P, k, wl.dtype)
    bufs = {
        "topk_idx": torch.empty((S, k), dtype=torch.int32, device=dev),
        "topk_w": torch.empty((S, k), dtype=torch.float32, device=dev),
        "m": torch.empty((N,), dtype=torch.float32, device=dev),
        "c_expert": torch.empty((N,), dtype=torch.int32, device=dev),
        "c_device": torch.empty((P,), dtype=torch.int32, device=dev),
        "loss": torch.empty((1,), dtype=torch.float32, device=dev),
        "send": torch.empty((S * k, d), dtype=x.dtype, device=dev),
        "slot": torch.empty((S, k), dtype=torch.int32, device=dev),
        "kept": torch.empty((N,), dtype=torch.int32, device=dev),
        "off": torch.empty((N + 1,), dtype=torch.int32, device=dev),
        "scd": torch.empty((P,), dtype=torch.int32, device=dev),
        "y": torch.empty((S, d), dtype=x.dtype, device=dev),
    }
    pen_d, cap_d = torch.from_numpy(pen).cuda(), torch.from_numpy(cap).cuda()

    def step(xin):
        b = bufs
        T.tamoe_gate(xin, w, P, k, None, b["topk_idx"], b["topk_w"], b["m"], b["c_expert"], b["c_device"], ws)
        T.tamoe_aux_loss(b["m"], b["c_expert"], pen_d, P, S, b["loss"])
        T.tamoe_dispatch(xin, b["topk_idx"], cap_d, N, P, b["send"], b["slot"], b["kept"], b["off"], b["scd"], ws)
        T.tamoe_combine(b["send"], S * k, b["slot"], b["topk_w"], b["y"])

    def fused_step(xin):
        b = bufs
        T.tamoe_gate_dispatch(xin, w, P, k, pen_d, cap_d, None, b["topk_idx"], b["topk_w"], b["m"], b["c_expert"],
                              b["c_device"], b["loss"], b["send"], b["slot"], b["kept"], b["off"], b["scd"], ws)
        T.tamoe_combine(b["send"], S * k, b["slot"], b["topk_w"], b["y"])

    if fused:
        step = fused_step
    x_in = x.clone()
    step(x_in)
    torch.cuda.synchronize()
    eager = {n: t.clone() for n, t in bufs.items()}
    K = int(eager["off"][-1].item())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step(x_in)
    for rep in range(3):
        for t in bufs.values():
            t.zero_()                      # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for n in bufs:
            a, b = eager[n], bufs[n]
            if n == "send":
                a, b = a[:K], b[:K]
            assert torch.equal(a.view(torch.uint8), b.view(torch.uint8)), (n, rep)
    # new input through the same graph: permuting the tokens permutes the routing
    perm = torch.randperm(S, device=dev)
    x_in.copy_(x[perm])
    g.replay()
    torch.cuda.synchronize()
    assert torch.equal(bufs["topk_idx"], eager["topk_idx"][perm])
    assert torch.equal(bufs["c_expert"], eager["c_expert"])


def test_bench_mix_probe_moves_the_rows_it_is_told_to():
    from paper_2302_09915_amd import bench_aids as B

    rows, d = 300, 512                                   # 1 KiB rows of bf16
    a = torch.randn((rows, d), device="cuda").to(torch.bfloat16)
    perm = torch.randperm(2 * rows, device="cuda").to(torch.int32)
    r0, r1 = perm[:rows].contiguous(), perm[rows:].contiguous()
    r1[7] = -1                                          # skipped
    b = torch.zeros((2 * rows, d), dtype=torch.bfloat16, device="cuda")
    B.mix_probe(a, b, r0, r1, 1)
    torch.cuda.synchronize()
    ai, bi = a.view(torch.int16), b.view(torch.int16)
    assert torch.equal(bi[r0.long()], ai)
    keep = r1 >= 0
    assert torch.equal(bi[r1[keep].long()], ai[keep])
    out = torch.empty_like(a)
    B.mix_probe(b, out, r0, r1, 2)
    torch.cuda.synchronize()
    expect = torch.where(keep[:, None], torch.zeros_like(ai), ai)   # x ^ x = 0 where both rows exist
    assert torch.equal(out.view(torch.int16), expect)
    with pytest.raises(RuntimeError):
        B.mix_probe(a[:, :100].contiguous(), b[:, :100].contiguous(), r0, r1, 1)
