#!/usr/bin/env python3
"""Benchmark of the TA-MoE hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens that are already in
HBM: tamoe_gate_dispatch (gate, loss, slots, scatter) -> tamoe_combine (identity expert: the
combine reads the send buffer); with --path separate: tamoe_gate -> tamoe_aux_loss ->
tamoe_dispatch -> tamoe_combine.  The metric is routed tokens per second.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large] [--cap-mode 0]

The timed region is `--blocks` blocks of K steps, each between two device synchronisations;
`value` and `ms_per_step` are those of the median block (min and max beside them).
Prints one JSON line.  Besides the contract fields it carries
  roofline     achieved algorithmic HBM GB/s of the longest-running kernel against 8 TB/s, from
               HIP events recorded around that kernel's launches inside the timed region;
  kernels      the same for every kernel of the step, from an untimed pass with events around
               every launch (two event records per launch cost ~3 us of GPU time each, so only
               the dominant kernel is bracketed while `value` is being measured);
  scatter      the row scatter twice: behind the gate (as in the step: part of x still sits in the
               last-level cache) and from HBM alone (tamoe_dispatch called on its own);
  other_workloads  ms per step of the paper-sized configurations, eager and replayed from a HIP graph;
  cpu_baseline the CPU oracle timed on the host cores on a bounded sample of the workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, vendor figure
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--blocks", type=int, default=5, help="timed blocks of --steps steps; the median block is reported")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large",
                    help="tiny, small, gpt_moe, skewed, large (the measured configurations) or one of the paper's own "
                         "shapes: paper_switch_fp16, paper_gshard_fp16, paper_switch_fp32, paper_gshard_fp32")
    ap.add_argument("--dtype", choices=["f32", "bf16", "f16"], default=None,
                    help="storage type instead of the workload's own (f16: the FP16 of the paper's GPT model table)")
    ap.add_argument("--cap-mode", type=int, default=0, help="0 uniform capacity, 1 proportional to the target pattern")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", "--no-backward", dest="no_extras", action="store_true",
                    help="skip the measurements beside the forward path (backward kernels, regrouping, variants, "
                         "the other workloads)")
    ap.add_argument("--no-trace", action="store_true",
                    help="no HIP events inside the timed region (per-kernel times then come from an extra traced pass)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (implies --no-trace)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="number of copies of (x, send, y) that the steps cycle through, so that a small workload's "
                         "rows come from HBM and not from the 256 MB last-level cache (default 1: same buffers)")
    ap.add_argument("--path", choices=["fused", "separate"], default="fused",
                    help="fused: tamoe_gate_dispatch + tamoe_combine (4 launches per step); separate: tamoe_gate, "
                         "tamoe_aux_loss, tamoe_dispatch, tamoe_combine (8 launches)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), as recorded in
    profiles/hbm_traffic.txt: lines `<workload> <kernel> <bytes>`, and the commit the counters were
    read at (its `# commit:` line).  (None, commit) if not recorded."""
    value, commit = None, None
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if line.startswith("# commit:") and len(parts) >= 3:
                    commit = parts[2]
                if len(parts) >= 3 and not line.startswith("#") and parts[0] == workload and parts[1] == kernel:
                    value = float(parts[2])
    except OSError:
        pass
    return value, commit


def cpu_baseline(wl, W, seconds: float):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import oracle

    # every host core this process may use: the machine's share set through OMP_NUM_THREADS where the
    # operator sets one (GPU machines hand a one-GPU job 16 cores), else all cores that are visible
    visible = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or visible
    threads = max(1, min(threads, oracle.max_threads()))
    oracle.set_threads(threads)
    beta, level = W.topology(wl)

    def run(S):
        inp = W.make_inputs(wl, S=S)
        steps = {}
        t_start = t0 = time.perf_counter()

        def lap(name):
            nonlocal t0
            t1 = time.perf_counter()
            steps[name] = round(t1 - t0, 4)
            t0 = t1

        c_hat, p, cap = oracle.setup(beta, level, wl.N, wl.rank, wl.k, S, wl.capacity_factor, 0)
        lap("setup")
        lg = oracle.logits(inp["x"], inp["w"], wl.dtype)
        lap("scores")
        r = oracle.route_from_logits(lg, wl.k, wl.P, p, cap)
        lap("softmax_topk_counts_losses_slots")
        send = oracle.scatter(inp["x"], wl.dtype, r["slot"], r["K"])
        lap("scatter")
        oracle.combine(send, wl.dtype, r["slot"], r["topk_w"], want_exact=False, want_rounded=True)
        lap("combine")
        return time.perf_counter() - t_start, steps

    probe_S = min(wl.S, 256)
    t_probe, _ = run(probe_S)
    S = int(min(wl.S, max(probe_S, seconds / max(t_probe, 1e-6) * probe_S)))
    S = max(64, S // 64 * 64) if wl.S >= 64 else wl.S
    t, steps = run(S)
    out = {"value": S / t, "unit": "tokens/s", "cores": threads, "host_cores_visible": visible,
           "cores_limited_by": "OMP_NUM_THREADS" if os.environ.get("OMP_NUM_THREADS") else "none", "kind": "oracle",
           "sample": f"first-draw sample of {S} of {wl.S} tokens of workload {wl.name}, whole path "
                     f"(setup, scores, softmax, top-k, counts, losses, slots, scatter, combine), {t:.2f} s",
           "per_step_seconds": steps}
    if threads > 1:
        # the same oracle on one thread, on a sample sized to a few seconds
        oracle.set_threads(1)
        S1 = int(min(S, max(probe_S, 4.0 / max(t, 1e-6) * S / threads)))
        S1 = max(64, S1 // 64 * 64) if wl.S >= 64 else wl.S
        t1, steps1 = run(S1)
        oracle.set_threads(threads)
        out["single_thread"] = {"value": S1 / t1, "unit": "tokens/s", "cores": 1,
                                "sample": f"first-draw sample of {S1} tokens, {t1:.2f} s", "per_step_seconds": steps1}
    return out


def _mean_us(ts) -> float:
    return float(np.mean(ts)) * 1e3


def _median_us(T, n_rec: int) -> float:
    return float(np.median([T.tamoe_trace_get(i)[1] for i in range(n_rec)])) * 1e3


def _rate(nbytes: float, us: float) -> dict:
    """Algorithmic bytes over time.  Not a measured HBM rate: bytes that a cache serves count too."""
    gbs = nbytes / (us * 1e-6) / 1e9
    return {"algo_bytes": int(nbytes), "algo_GBs": round(gbs, 1), "algo_frac_of_peak": round(gbs / HBM_PEAK_GBS, 4)}


def _timed_us(torch, fn, reps: int = 5) -> float:
    """Median duration of fn() in microseconds, from events on the current stream (the stream fn enqueues on)."""
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return float(np.median([a.elapsed_time(b) for a, b in ev])) * 1e3


class Path:
    """The buffers of one workload on the device and one step of the path over them."""

    def __init__(self, T, W, torch, wl, cap_mode: int, rotate: int, fused: bool = True):
        self.T, self.W, self.torch, self.wl = T, W, torch, wl
        self.fused = fused
        self.dev = dev = torch.device("cuda:0")
        torch.cuda.set_device(dev)
        inp = W.make_inputs(wl)
        self.beta, self.level = W.topology(wl)
        _, pen, cap = T.tamoe_topo_pattern(self.beta, self.level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor,
                                           cap_mode)
        self.x, self.w = self._upload(inp["x"]), self._upload(inp["w"])
        S, d, N, P, k = wl.S, wl.d, wl.N, wl.P, wl.k
        self.row_bytes = d * wl.elem_bytes
        i32, f32 = torch.int32, torch.float32
        self.pen = torch.from_numpy(pen).to(dev)
        self.cap = torch.from_numpy(cap).to(dev)
        self.ws = T.workspace(S, d, N, P, k, wl.dtype, dev)
        self.topk_idx = torch.empty((S, k), dtype=i32, device=dev)
        self.topk_w = torch.empty((S, k), dtype=f32, device=dev)
        self.m = torch.empty((N,), dtype=f32, device=dev)
        self.c_expert = torch.empty((N,), dtype=i32, device=dev)
        self.c_device = torch.empty((P,), dtype=i32, device=dev)
        self.loss = torch.empty((1,), dtype=f32, device=dev)
        self.send = torch.empty((S * k, d), dtype=self.x.dtype, device=dev)
        self.slot = torch.empty((S, k), dtype=i32, device=dev)
        self.kept = torch.empty((N,), dtype=i32, device=dev)
        self.off = torch.empty((N + 1,), dtype=i32, device=dev)
        self.scd = torch.empty((P,), dtype=i32, device=dev)
        self.y = torch.empty((S, d), dtype=self.x.dtype, device=dev)
        self.rotate = rotate
        self.sets = [(self.x, self.send, self.y)] + [
            (self.x.clone(), torch.empty_like(self.send), torch.empty_like(self.y)) for _ in range(rotate - 1)]
        self.turn = 0
        self._bound = None

    def _upload(self, a):
        t = self.torch.from_numpy(a)
        if self.wl.dtype == self.W.BF16:
            t = t.view(self.torch.int16).view(self.torch.bfloat16)
        elif self.wl.dtype == self.W.F16:
            t = t.view(self.torch.int16).view(self.torch.float16)
        return t.to(self.dev)

    def step(self):
        T, wl = self.T, self.wl
        xs, sends, ys = self.sets[self.turn % self.rotate]
        self.turn += 1
        # stream=None: the binding passes torch's current stream (the capture stream under --graph)
        if self.fused:
            T.tamoe_gate_dispatch(xs, self.w, wl.P, wl.k, self.pen, self.cap, None, self.topk_idx, self.topk_w, self.m,
                                  self.c_expert, self.c_device, self.loss, sends, self.slot, self.kept, self.off,
                                  self.scd, self.ws, None)
            T.tamoe_combine(sends, wl.S * wl.k, self.slot, self.topk_w, ys, None)
            return
        T.tamoe_gate(xs, self.w, wl.P, wl.k, None, self.topk_idx, self.topk_w, self.m, self.c_expert, self.c_device,
                     self.ws, None)
        T.tamoe_aux_loss(self.m, self.c_expert, self.pen, wl.P, wl.S, self.loss, None)
        T.tamoe_dispatch(xs, self.topk_idx, self.cap, wl.N, wl.P, sends, self.slot, self.kept, self.off, self.scd,
                         self.ws, None)
        # identity expert: the rows come back as they were sent; S*k bounds the row count
        T.tamoe_combine(sends, wl.S * wl.k, self.slot, self.topk_w, ys, None)

    def step_bound(self):
        """The same step through calls whose arguments were marshalled once (T.bind): what a loop over
        fixed buffers would use, so that a small workload is timed on the device and not on the Python
        side of the binding.  Not for use under stream capture (the stream is fixed when binding)."""
        if self._bound is None:
            T, wl = self.T, self.wl
            self._bound = []
            for xs, sends, ys in self.sets:
                if self.fused:
                    calls = [T.bind(T.tamoe_gate_dispatch, xs, self.w, wl.P, wl.k, self.pen, self.cap, None,
                                    self.topk_idx, self.topk_w, self.m, self.c_expert, self.c_device, self.loss, sends,
                                    self.slot, self.kept, self.off, self.scd, self.ws, None)]
                else:
                    calls = [T.bind(T.tamoe_gate, xs, self.w, wl.P, wl.k, None, self.topk_idx, self.topk_w, self.m,
                                    self.c_expert, self.c_device, self.ws, None),
                             T.bind(T.tamoe_aux_loss, self.m, self.c_expert, self.pen, wl.P, wl.S, self.loss, None),
                             T.bind(T.tamoe_dispatch, xs, self.topk_idx, self.cap, wl.N, wl.P, sends, self.slot,
                                    self.kept, self.off, self.scd, self.ws, None)]
                calls.append(T.bind(T.tamoe_combine, sends, wl.S * wl.k, self.slot, self.topk_w, ys, None))
                self._bound.append(calls)
        calls = self._bound[self.turn % self.rotate]
        self.turn += 1
        for c in calls:
            c()

    def sync(self):
        self.torch.cuda.synchronize()

    def kept_rows(self) -> int:
        return int(self.off[-1].item())

    def live_tokens(self) -> int:
        return int((self.slot >= 0).any(dim=1).sum().item())

    def collect(self) -> dict:
        """Stops the trace; kernel name -> list of durations in ms."""
        out = {}
        for i in range(self.T.tamoe_trace_stop()):
            name, ms = self.T.tamoe_trace_get(i)
            out.setdefault(name, []).append(ms)
        return out


def measure_probes(p: Path):
    """Yardsticks outside the timed region (kernels of libtamoe_bench.so, not of the product library):
    a plain copy of x into y, and (k = 2, rows a multiple of 1 KiB) the scatter's and the combine's bare
    memory operations on the realised slot table."""
    from paper_2302_09915_amd import bench_aids as B

    wl, torch = p.wl, p.torch
    S, k, row = wl.S, wl.k, p.row_bytes
    B.copy_probe(p.x, p.y)
    copy_us = _timed_us(torch, lambda: B.copy_probe(p.x, p.y))
    copy_gbs = 2.0 * S * row / (copy_us * 1e-6) / 1e9
    copy = {"bytes_moved": int(2 * S * row), "median_us": round(copy_us, 2), "GBs": round(copy_gbs, 1),
            "frac_of_hbm_peak": round(copy_gbs / HBM_PEAK_GBS, 4)}
    mix = None
    if k == 2 and row % 1024 == 0:
        r0 = p.slot[:, 0].contiguous()
        r1 = p.slot[:, 1].contiguous()
        B.mix_probe(p.x, p.send, r0, r1, 1)
        sc_us = _timed_us(torch, lambda: B.mix_probe(p.x, p.send, r0, r1, 1))
        ga_us = _timed_us(torch, lambda: B.mix_probe(p.send, p.y, r0, r1, 2))
        K0 = int((p.slot >= 0).sum().item())
        mix = {"scatter_1r2w": {"median_us": round(sc_us, 2),
                                "GBs": round((p.live_tokens() + K0) * row / (sc_us * 1e-6) / 1e9, 1)},
               "gather_2r1w": {"median_us": round(ga_us, 2), "GBs": round((K0 + S) * row / (ga_us * 1e-6) / 1e9, 1)}}
    return copy, mix


def measure_scatter_from_hbm(p: Path, nbytes: int):
    """The scatter with every row of x coming from HBM: tamoe_dispatch on its own, back to back (its
    loads and stores are streaming ones, so nothing of x stays in the last-level cache between calls).
    In the step the scatter runs behind the gate, which leaves part of x in that cache."""
    T, wl = p.T, p.wl
    for _ in range(2):
        T.tamoe_dispatch(p.x, p.topk_idx, p.cap, wl.N, wl.P, p.send, p.slot, p.kept, p.off, p.scd, p.ws, None)
    p.sync()
    T.tamoe_trace_filter("dispatch_copy_kernel")
    T.tamoe_trace_start(10)
    for _ in range(10):
        T.tamoe_dispatch(p.x, p.topk_idx, p.cap, wl.N, wl.P, p.send, p.slot, p.kept, p.off, p.scd, p.ws, None)
    p.sync()
    rec = p.collect()
    T.tamoe_trace_filter(None)
    T.tamoe_trace_clear()
    us = _mean_us(rec["dispatch_copy_kernel"])
    return {"kernel": "dispatch_copy_kernel", "avg_us": round(us, 2), **_rate(nbytes, us)}


def measure_workload(T, W, torch, name: str, steps: int, blocks: int = 3):
    """ms per step of another configuration: eager and replayed from a HIP graph (median block)."""
    wl = W.workload(name)
    p = Path(T, W, torch, wl, 0, 1, fused=True)
    out = {"S": wl.S, "d": wl.d, "N": wl.N, "k": wl.k}
    for _ in range(5):
        p.step()
    p.sync()

    def median_ms(run):
        ts = []
        for _ in range(blocks):
            p.sync()
            t0 = time.perf_counter()
            for _ in range(steps):
                run()
            p.sync()
            ts.append((time.perf_counter() - t0) * 1e3 / steps)
        return round(float(np.median(ts)), 4)

    out["eager_ms_per_step"] = median_ms(p.step_bound)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        p.step()
    for _ in range(2):
        graph.replay()
    out["graph_ms_per_step"] = median_ms(graph.replay)
    out["tokens_per_s_graph"] = round(wl.S / (out["graph_ms_per_step"] * 1e-3), 1)
    return out


def measure_other_mode(p: Path, cap_mode: int, steps: int):
    """The other capacity mode beside the headline one (uniform <-> proportional to the target
    pattern): a short timed region of its own on the same buffers; the headline state is restored."""
    T, wl, torch = p.T, p.wl, p.torch
    K_main = p.kept_rows()
    _, _, cap_o = T.tamoe_topo_pattern(p.beta, p.level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor,
                                       1 - cap_mode)
    cap_keep = p.cap.clone()
    p.cap.copy_(torch.from_numpy(cap_o).to(p.dev))
    n = max(1, min(steps, 20))
    for _ in range(2):
        p.step()
    p.sync()
    t0 = time.perf_counter()
    for _ in range(n):
        p.step()
    p.sync()
    elapsed = time.perf_counter() - t0
    K_o = p.kept_rows()
    p.cap.copy_(cap_keep)
    for _ in range(p.rotate):                    # slot, send and the size outputs are those of the headline mode again
        p.step()
    p.sync()
    assert p.kept_rows() == K_main
    return {"cap_mode": 1 - cap_mode, "steps": n, "ms_per_step": round(elapsed * 1e3 / n, 4),
            "value": round(wl.S * n / elapsed, 1), "unit": "tokens/s", "kept_rows_K": K_o,
            "drop_rate": round(1.0 - K_o / (wl.S * wl.k), 4)}


def measure_backward(p: Path):
    """Backward kernels: a pass of their own with events around every launch; not part of `value`."""
    T, wl, torch = p.T, p.wl, p.torch
    S, d, N, P, k, row = wl.S, wl.d, wl.N, wl.P, wl.k, p.row_bytes
    K_now = p.kept_rows()
    logits = torch.empty((S, N), dtype=torch.float32, device=p.dev)
    T.tamoe_gate(p.x, p.w, P, k, logits, p.topk_idx, p.topk_w, p.m, p.c_expert, p.c_device, p.ws, None)
    dy = p.y                                     # any tensor of the shape of y serves as upstream gradient
    d_recv = torch.empty((max(K_now, 1), d), dtype=p.x.dtype, device=p.dev)
    d_w = torch.empty((S, k), dtype=torch.float32, device=p.dev)
    d_logits = torch.empty((S, N), dtype=torch.float32, device=p.dev)
    d_x = torch.empty((S, d), dtype=p.x.dtype, device=p.dev)

    def bwd():
        T.tamoe_combine_bwd(dy, p.send, K_now, p.slot, p.topk_w, d_recv, d_w, None)
        T.tamoe_gate_bwd(logits, p.topk_idx, d_w, p.pen, p.c_expert, 1.0, P, d_logits, None)
        T.tamoe_dispatch_bwd(d_recv, K_now, p.slot, d_x, None)

    for _ in range(3):
        bwd()
    p.sync()
    reps = 10
    T.tamoe_trace_start(3 * reps)
    for _ in range(reps):
        bwd()
    p.sync()
    rec = p.collect()
    T.tamoe_trace_clear()
    nbytes = {"combine_bwd_kernel": S * row + 2 * K_now * row + S * k * 12,
              "gate_bwd_kernel": 2 * S * N * 4 + S * k * 8,
              "dispatch_bwd_kernel": K_now * row + S * row + S * k * 4}
    return [{"kernel": name, "avg_us": round(_mean_us(ts), 2), **_rate(nbytes[name], _mean_us(ts))}
            for name, ts in rec.items()]


def measure_regroup(p: Path):
    """Receive-side regrouping: the kept rows of `send` stand in for a receive buffer with P source
    chunks x E local experts (E = 2 when the workload has one expert per device, where regrouping is
    the identity), seeded Poisson segment sizes.  Not part of `value`."""
    T, wl, torch = p.T, p.wl, p.torch
    E_r = wl.E if wl.E > 1 else 2
    P_r = min(wl.P, 128 // E_r)
    rows = p.kept_rows()
    if rows < P_r * E_r:
        return None
    rng = np.random.Generator(np.random.Philox(key=[wl.seed, 11]))
    share = rng.poisson(64, size=(P_r, E_r)).astype(np.float64) + 1.0
    cnt = np.floor(share / share.sum() * rows).astype(np.int32)
    cnt[0, 0] += rows - int(cnt.sum())
    cnt_d = torch.from_numpy(cnt).to(p.dev)
    rin = p.send[:rows]
    rout = torch.empty_like(rin)
    for _ in range(2):
        T.tamoe_regroup(rin, cnt_d, True, rout, None, p.ws, None)
    p.sync()
    T.tamoe_trace_filter("regroup_copy_kernel")
    T.tamoe_trace_start(10)
    for _ in range(10):
        T.tamoe_regroup(rin, cnt_d, True, rout, None, p.ws, None)
    p.sync()
    rec = p.collect()
    T.tamoe_trace_filter(None)
    T.tamoe_trace_clear()
    us = _mean_us(rec["regroup_copy_kernel"])
    return {"kernel": "regroup_copy_kernel", "P": P_r, "E": E_r, "rows": rows, "avg_us": round(us, 2),
            **_rate(2 * rows * p.row_bytes, us)}


def measure_variants(p: Path):
    """The fixed-size zero-padded layout against the packed one (rows written, time of the row
    movers) and the weight renormalisation.  Not part of `value`."""
    T, wl, torch = p.T, p.wl, p.torch
    S, d, N, P, k, row = wl.S, wl.d, wl.N, wl.P, wl.k, p.row_bytes
    C = int(p.cap.max().item())
    pad_rows = N * C
    send_p = torch.empty((pad_rows, d), dtype=p.x.dtype, device=p.dev)
    slot_p = torch.empty_like(p.slot)
    kept_p = torch.empty_like(p.kept)
    w_n = torch.empty_like(p.topk_w)
    d_wn = torch.empty_like(p.topk_w)

    def var():
        T.tamoe_dispatch_padded(p.x, p.topk_idx, p.cap, N, P, C, send_p, slot_p, kept_p, p.ws, None)
        T.tamoe_renorm_topk(p.topk_w, w_n, None)
        T.tamoe_renorm_topk_bwd(p.topk_w, w_n, d_wn, None)

    for _ in range(2):
        var()
    p.sync()
    reps = 10
    T.tamoe_trace_start(7 * reps)
    for _ in range(reps):
        var()
    p.sync()
    us = {n: _mean_us(ts) for n, ts in p.collect().items()}
    T.tamoe_trace_clear()
    K_p = int(kept_p.sum().item())
    live_p = int((slot_p >= 0).any(dim=1).sum().item())
    mover_us = us["dispatch_copy_kernel"] + us["dispatch_pad_fill_kernel"]
    mover_bytes = (live_p + pad_rows) * row + S * k * 8
    return {
        "padded_dispatch": {"C": C, "rows_written": pad_rows, "rows_kept": K_p,
                            "copy_us": round(us["dispatch_copy_kernel"], 2),
                            "pad_fill_us": round(us["dispatch_pad_fill_kernel"], 2),
                            "algo_bytes": int(mover_bytes),
                            "achieved_GBs": round(mover_bytes / (mover_us * 1e-6) / 1e9, 1),
                            "rows_vs_packed": round(pad_rows / max(K_p, 1), 4)},
        "renorm_topk_us": round(us["renorm_topk_kernel"], 2),
        "renorm_topk_bwd_us": round(us["renorm_topk_bwd_kernel"], 2),
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; the exchange between devices is out of scope "
              "(--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2302_09915_amd as T
    import tamoe_workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    T.lib()
    wl = W.workload(args.workload)
    if args.dtype is not None:
        import dataclasses

        wl = dataclasses.replace(wl, dtype={"f32": W.F32, "bf16": W.BF16, "f16": W.F16}[args.dtype])
    p = Path(T, W, torch, wl, args.cap_mode, max(1, args.rotate), fused=args.path == "fused")
    S, N, k, row = wl.S, wl.N, wl.k, p.row_bytes

    for _ in range(max(args.warmup, 0)):
        p.step()
    p.sync()
    copy_probe, mix_probe = measure_probes(p)

    # Pass 1 (not timed): every launch bracketed by HIP events -> the per-kernel table and the name
    # of the longest-running kernel.  Two event records per launch cost ~3 us of GPU time each, so
    # this pass is kept out of `value`.
    launches_per_step = 10
    table_steps = max(1, min(args.steps, 20))
    T.tamoe_trace_filter(None)
    T.tamoe_trace_start(launches_per_step * table_steps)
    for _ in range(table_steps):
        p.step()
    p.sync()
    per_kernel = p.collect()
    dominant = max(per_kernel, key=lambda n: float(np.mean(per_kernel[n])))

    run_step = p.step_bound
    if args.graph:
        # the library only enqueues kernels on the current stream, so a step can be captured as is
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            p.step()                             # with --rotate the replays reuse the captured set
        run_step = graph.replay
        for _ in range(2):
            run_step()
        p.sync()

    # Pass 2, the timed region: `blocks` blocks of K steps, each between two synchronisations; only the
    # dominant kernel is bracketed by events (two records per step), which is what `roofline.achieved`
    # is computed from.  The median block gives `value`.
    traced_in_timed_region = not (args.no_trace or args.graph)
    n_blocks = max(1, args.blocks)
    if traced_in_timed_region:
        T.tamoe_trace_filter(dominant)
        T.tamoe_trace_start(args.steps * n_blocks)
    block_s = []
    for _ in range(n_blocks):
        p.sync()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_step()
        p.sync()
        block_s.append(time.perf_counter() - t0)
    elapsed = float(np.median(block_s))
    dominant_live = p.collect().get(dominant) if traced_in_timed_region else None
    T.tamoe_trace_filter(None)
    T.tamoe_trace_clear()

    other_mode = None if args.graph else measure_other_mode(p, args.cap_mode, args.steps)
    extras = not args.no_extras
    backward = measure_backward(p) if extras else None
    regroup = measure_regroup(p) if extras else None
    variants = measure_variants(p) if extras else None

    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = S * args.steps / elapsed

    # realised routing (for the algorithmic byte counts)
    K = p.kept_rows()
    live_tokens = p.live_tokens()
    algo_bytes = {
        "gate_bf16_kernel": S * row + N * row + S * k * 8,
        "gate_f16_kernel": S * row + N * row + S * k * 8,
        "gate_f32_kernel": S * row + N * row + S * k * 8,
        "select_kernel": S * N * 4 + S * k * 8,
        "dispatch_copy_kernel": live_tokens * row + K * row + S * k * 8,
        "route_copy_kernel": live_tokens * row + K * row + S * k * 12,
        "combine_kernel": K * row + S * row + S * k * 8,
    }
    kernels = []
    for name, ts in per_kernel.items():
        entry = {"kernel": name, "launches": len(ts), "avg_us": round(_mean_us(ts), 2)}
        if name in algo_bytes:
            entry.update(_rate(algo_bytes[name], _mean_us(ts)))
        kernels.append(entry)
    kernels.sort(key=lambda e: -e["avg_us"])
    roofline = None
    if dominant in algo_bytes:
        live = dominant_live if dominant_live else per_kernel[dominant]
        dom_us = _mean_us(live)
        gbs = algo_bytes[dominant] / (dom_us * 1e-6) / 1e9
        traffic, traffic_commit = measured_traffic(wl.name, dominant)
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                    "traffic": traffic,
                    "traffic_from": f"profiles/hbm_traffic.txt (rocprofv3 --pmc, counters read at commit {traffic_commit})",
                    "algo_bytes_per_launch": int(algo_bytes[dominant]), "avg_launch_us": round(dom_us, 2),
                    "launches_timed": len(live),
                    "timed_in": "timed region" if dominant_live else "table pass"}

    # the scatter twice: as it runs in the step (behind the gate) and with x from HBM alone
    scatter = None
    scatter_name = next((n for n in ("route_copy_kernel", "dispatch_copy_kernel") if n in per_kernel), None)
    if scatter_name is not None and not args.graph:
        us = _mean_us(per_kernel[scatter_name])
        scatter = {"behind_gate": {"kernel": scatter_name, "avg_us": round(us, 2), **_rate(algo_bytes[scatter_name], us),
                                   "note": "part of x is served by the 256 MB last-level cache that the gate left it in"},
                   "from_hbm": measure_scatter_from_hbm(p, algo_bytes["dispatch_copy_kernel"])}
    others = None
    if extras and not args.graph:
        others = {n: measure_workload(T, W, torch, n, 50) for n in ("gpt_moe", "skewed", "small", "tiny") if n != wl.name}

    total_algo = algo_bytes["gate_bf16_kernel"] \
        + algo_bytes["dispatch_copy_kernel"] + algo_bytes["combine_kernel"]

    result = {
        "metric": "routed tokens/sec (gate+aux_loss+dispatch+combine), 1 GPU",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "blocks": n_blocks,
        "ms_per_step_min": round(min(block_s) * 1e3 / args.steps, 4),
        "ms_per_step_max": round(max(block_s) * 1e3 / args.steps, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": {W.F32: "f32", W.BF16: "bf16", W.F16: "f16"}[wl.dtype],
        "data": "synthetic",
        "config": {"workload": wl.name, "S": S, "d": wl.d, "N": N, "k": k, "P": wl.P, "E": wl.E,
                   "capacity_factor": wl.capacity_factor, "cap_mode": args.cap_mode,
                   "topology": f"{wl.nodes}x{wl.devs_per_node} ratio {wl.bw_ratio:g}:1", "rank": wl.rank,
                   "kept_rows_K": K, "tokens_with_a_kept_choice": live_tokens,
                   "drop_rate": round(1.0 - K / (S * k), 4), "rotating_buffer_sets": p.rotate},
        "path_algo_bytes_per_step": int(total_algo),
        "path_achieved_GBs": round(total_algo / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "copy_probe": copy_probe,
        "mix_probe": mix_probe,
        "kernels": kernels,
        "kernels_note": "algo_GBs = algorithmic bytes / kernel time (bytes that a cache serves count too); "
                        "avg_us from the untimed pass with events around every launch",
        "scatter": scatter,
        "other_workloads": others,
        "backward_kernels": backward,
        "regroup_kernel": regroup,
        "variants": variants,
        "other_capacity_mode": other_mode,
        "l_topo": float(p.loss.item()),
        "mode": "graph replay" if args.graph else "eager",
        "path": args.path,
        "kernels_table_from": f"untimed pass of {table_steps} steps with HIP events around every launch",
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, W, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
