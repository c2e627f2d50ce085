"""Seeded synthetic inputs for the TA-MoE hot path (numpy only).

This module is the one piece that both the HIP path's tests/bench and the CPU
oracle's tests are allowed to share.  It holds no arithmetic of the method:
it only draws random tensors of the shapes the paper's GPT-MoE workloads have
(Evaluation, "Experiment setup" and the GPT model table: hidden size 1024,
8..64 experts, one expert per device, Switch top-1 / GShard top-2), builds the
two-tier inverse-bandwidth table of a virtual symmetric tree (Section 3.2
"Network Topology": nodes x devices, intra-node links faster than inter-node),
and rounds values to the storage type.  The paper's training data
(openwebtext2 activations) is not available; these tensors stand in for it.

Every draw comes from numpy's counter-based Philox generator keyed by the
config's seed, so the same bytes are produced on every machine.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

F32 = 0
BF16 = 1
F16 = 2      # IEEE half precision, the data type of the paper's cluster-A runs (GPT model table)


@dataclass(frozen=True)
class Workload:
    """One synthetic MoE-layer call on a single device (rank) of a virtual cluster."""

    name: str
    S: int            # tokens on this device
    d: int            # hidden size
    dtype: int        # F32, BF16 or F16 storage of x, W and y
    N: int            # experts
    k: int            # experts selected per token
    capacity_factor: float
    nodes: int        # virtual topology: nodes x devs_per_node devices
    devs_per_node: int
    bw_ratio: float   # intra-node bandwidth / inter-node bandwidth
    seed: int
    zipf_s: Optional[float] = None  # if set, expert popularity ~ Zipf(s) through a bias feature
    rank: int = 0

    @property
    def P(self) -> int:
        return self.nodes * self.devs_per_node

    @property
    def E(self) -> int:
        return self.N // self.P

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == F32 else 2


# The five configurations the build is measured on.  Seeds: 0 for Tiny (given),
# then the config index.
WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", S=512, d=64, dtype=F32, N=8, k=1, capacity_factor=1.0,
                     nodes=2, devs_per_node=4, bw_ratio=4.0, seed=0),
    "small": Workload("small", S=4096, d=512, dtype=BF16, N=16, k=2, capacity_factor=1.25,
                      nodes=4, devs_per_node=4, bw_ratio=8.0, seed=1),
    "gpt_moe": Workload("gpt_moe", S=16384, d=1024, dtype=BF16, N=64, k=2, capacity_factor=1.2,
                        nodes=8, devs_per_node=8, bw_ratio=10.0, seed=2),
    "skewed": Workload("skewed", S=16384, d=2048, dtype=BF16, N=64, k=1, capacity_factor=1.0,
                       nodes=8, devs_per_node=8, bw_ratio=16.0, seed=3, zipf_s=1.2),
    "large": Workload("large", S=65536, d=4096, dtype=BF16, N=128, k=2, capacity_factor=1.25,
                      nodes=8, devs_per_node=8, bw_ratio=12.0, seed=4),
}


# The shapes of the paper's own runs (Evaluation, GPT model table: hidden size 1024, Switch top-1 with
# capacity factor 1.0 and GShard top-2 with 2.0 in FP16 on its first cluster, both gates with 1.2 in
# FP32 on the other two; batch size 6 resp. 4 sequences per device, taken at 1024 tokens each; up to 64
# experts, one per device, 8 devices per node).  Not among the five measured configurations: extra
# shapes for the benchmark and one parity test each.  The bandwidth ratio is the GPT-MoE config's.
PAPER_SHAPES: Dict[str, Workload] = {
    "paper_switch_fp16": Workload("paper_switch_fp16", S=6144, d=1024, dtype=F16, N=64, k=1, capacity_factor=1.0,
                                  nodes=8, devs_per_node=8, bw_ratio=10.0, seed=11),
    "paper_gshard_fp16": Workload("paper_gshard_fp16", S=6144, d=1024, dtype=F16, N=64, k=2, capacity_factor=2.0,
                                  nodes=8, devs_per_node=8, bw_ratio=10.0, seed=12),
    "paper_switch_fp32": Workload("paper_switch_fp32", S=4096, d=1024, dtype=F32, N=64, k=1, capacity_factor=1.2,
                                  nodes=8, devs_per_node=8, bw_ratio=10.0, seed=13),
    "paper_gshard_fp32": Workload("paper_gshard_fp32", S=4096, d=1024, dtype=F32, N=64, k=2, capacity_factor=1.2,
                                  nodes=8, devs_per_node=8, bw_ratio=10.0, seed=14),
}


def workload(name: str) -> Workload:
    """A measured configuration or one of the paper's own shapes, by name."""
    if name in WORKLOADS:
        return WORKLOADS[name]
    if name in PAPER_SHAPES:
        return PAPER_SHAPES[name]
    raise KeyError(f"unknown workload {name!r}; known: {sorted(WORKLOADS) + sorted(PAPER_SHAPES)}")


# ----------------------------------------------------------------------------
# storage-type helpers (bit manipulation only)
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 values to bfloat16 (nearest, ties to even); returns uint16 bit patterns.

    Inputs must be finite (the generators only produce finite values)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns (uint16) to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a: np.ndarray, dtype: int) -> np.ndarray:
    """float32 array -> the array that is handed to both sides (float32, or uint16 bit patterns of
    bfloat16 / half precision values)."""
    if dtype == F32:
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == F16:
        return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)
    return f32_to_bf16_bits(a)


def storage_to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    """Exact values of a storage buffer as float64 (for test-side inspection only)."""
    if dtype == F32:
        return a.astype(np.float64)
    if dtype == F16:
        return np.ascontiguousarray(a, dtype=np.uint16).view(np.float16).astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


# ----------------------------------------------------------------------------
# random tensors
# ----------------------------------------------------------------------------

def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def _normal_storage(rng: np.random.Generator, rows: int, cols: int, scale: float, dtype: int,
                    chunk_rows: int = 8192) -> np.ndarray:
    out = np.empty((rows, cols), dtype=np.float32 if dtype == F32 else np.uint16)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        blk = rng.standard_normal((r1 - r0, cols), dtype=np.float32)
        if scale != 1.0:
            blk *= np.float32(scale)
        out[r0:r1] = to_storage(blk, dtype)
    return out


def zipf_popularity(N: int, s: float) -> np.ndarray:
    """Target expert popularity: share of expert e proportional to (e+1)^-s."""
    w = 1.0 / np.power(np.arange(1, N + 1, dtype=np.float64), s)
    return w / w.sum()


def zipf_bias(N: int, s: float, seed: int, draws: int = 1 << 15, iters: int = 80) -> np.ndarray:
    """Per-expert additive offsets b[e] such that, for i.i.d. standard normal scores g,
    the index of the largest g[e] + b[e] is distributed close to Zipf(s) over e.

    Calibrated on `draws` synthetic normal score vectors from a stream of their own (not on the
    token matrix): a fixed number of damped log-ratio updates b += 0.25 * (log(target) -
    log(observed share)); the damping keeps the update stable where a normal tail makes the share
    of a rare expert very sensitive to its offset.
    The result is a recipe for an input tensor; the realised popularity on the real tokens is
    approximate by construction and is reported by the bench."""
    target = zipf_popularity(N, s)
    g = _rng(seed, 7).standard_normal((draws, N), dtype=np.float32).astype(np.float64)
    b = np.log(target)
    b -= b.max()
    for _ in range(iters):
        share = np.bincount(np.argmax(g + b, axis=1), minlength=N).astype(np.float64)
        share = (share + 0.5) / (draws + 0.5 * N)
        b += 0.25 * (np.log(target) - np.log(share))
        b -= b.max()
    return b


def make_inputs(wl: Workload, S: Optional[int] = None) -> Dict[str, np.ndarray]:
    """Token matrix x[S,d] ~ N(0,1) and gate weight W[N,d] ~ N(0,1/d) in wl.dtype storage.

    For a Zipf workload the last feature of every token is the constant 1 and the last column
    of W carries the popularity offsets, so the gate stays a pure linear map (no bias term).
    `S` overrides the token count (the first S rows of the full tensor are NOT guaranteed to be
    reproduced; a different S is a different draw of the same distribution)."""
    S = wl.S if S is None else int(S)
    x = _normal_storage(_rng(wl.seed, 0), S, wl.d, 1.0, wl.dtype)
    w32 = _rng(wl.seed, 1).standard_normal((wl.N, wl.d), dtype=np.float32)
    w32 *= np.float32(1.0 / np.sqrt(wl.d))
    if wl.zipf_s is not None:
        one = to_storage(np.ones((1,), dtype=np.float32), wl.dtype)[0]
        x[:, wl.d - 1] = one
        w32[:, wl.d - 1] = zipf_bias(wl.N, wl.zipf_s, wl.seed).astype(np.float32)
    w = to_storage(w32, wl.dtype)
    return {"x": x, "w": w}


# ----------------------------------------------------------------------------
# virtual topology tables
# ----------------------------------------------------------------------------

def two_tier_topology(nodes: int, devs_per_node: int, bw_ratio: float):
    """Inverse-bandwidth table beta[P,P] and tree-level table level[P,P] of a 2-layer symmetric
    tree: devices of one node share a switch (level 0, beta = 1, the diagonal included),
    devices of different nodes talk through the slower tier (level 1, beta = bw_ratio)."""
    P = nodes * devs_per_node
    node = np.arange(P) // devs_per_node
    level = (node[:, None] != node[None, :]).astype(np.int32)
    beta = np.where(level == 0, 1.0, float(bw_ratio)).astype(np.float64)
    return beta, level


def topology(wl: Workload):
    return two_tier_topology(wl.nodes, wl.devs_per_node, wl.bw_ratio)


def noisy_topology(nodes: int, devs_per_node: int, bw_ratio: float, seed: int, rel_noise: float = 0.05):
    """A 'profiled' table: the two-tier beta with multiplicative noise on every entry
    (what smoothing per tree level is meant to average out)."""
    beta, level = two_tier_topology(nodes, devs_per_node, bw_ratio)
    r = _rng(seed, 3).uniform(1.0 - rel_noise, 1.0 + rel_noise, size=beta.shape)
    return beta * r, level


def random_logits(seed: int, S: int, N: int, ties: bool = False) -> np.ndarray:
    """float32 score matrix for feeding the selection stage directly.  With ties=True the scores
    are drawn from a handful of values so that equal scores are frequent."""
    rng = _rng(seed, 5)
    if ties:
        return rng.integers(-2, 3, size=(S, N)).astype(np.float32) * np.float32(0.5)
    return rng.standard_normal((S, N), dtype=np.float32) * np.float32(2.0)


def random_routing(seed: int, S: int, N: int, k: int, skew: float = 0.0) -> np.ndarray:
    """int32 topk_idx[S,k] with distinct experts per token, for feeding dispatch directly.
    skew > 0 makes low-numbered experts more popular."""
    rng = _rng(seed, 6)
    score = rng.standard_normal((S, N))
    if skew > 0.0:
        score = score - skew * np.log1p(np.arange(N, dtype=np.float64))[None, :]
    order = np.argsort(-score, axis=1, kind="stable")[:, :k]
    return np.ascontiguousarray(order.astype(np.int32))
