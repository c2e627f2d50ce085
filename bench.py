#!/usr/bin/env python3
"""Benchmark of the TA-MoE hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic tokens that are already in
HBM: tamoe_gate -> tamoe_aux_loss -> tamoe_dispatch -> tamoe_combine (identity expert: the
combine reads the send buffer).  The metric is routed tokens per second.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large] [--cap-mode 0]

Prints one JSON line.  Besides the contract fields it carries
  roofline     achieved algorithmic HBM GB/s of the longest-running kernel against 8 TB/s, from
               HIP events recorded around that kernel's launches inside the timed region;
  kernels      the same for every kernel of the step, from an untimed pass with events around
               every launch (two event records per launch cost ~3 us of GPU time each, so only
               the dominant kernel is bracketed while `value` is being measured);
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
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--cap-mode", type=int, default=0, help="0 uniform capacity, 1 proportional to the target pattern")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-backward", action="store_true", help="skip the (untimed) measurement of the backward kernels")
    ap.add_argument("--no-trace", action="store_true",
                    help="no HIP events inside the timed region (per-kernel times then come from an extra traced pass)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (implies --no-trace)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="number of copies of (x, send, y) that the steps cycle through, so that a small workload's "
                         "rows come from HBM and not from the 256 MB last-level cache (default 1: same buffers)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE), as recorded in
    profiles/hbm_traffic.txt: lines `<workload> <kernel> <bytes>`.  None if not recorded."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and not line.startswith("#") and parts[0] == workload and parts[1] == kernel:
                    return float(parts[2])
    except OSError:
        pass
    return None


def cpu_baseline(wl, W, seconds: float):
    """The oracle, as it stands, on a bounded sample of the same workload."""
    import oracle

    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or min(16, os.cpu_count() or 1)
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
    out = {"value": S / t, "unit": "tokens/s", "cores": threads, "kind": "oracle",
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
    wl = W.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    inp = W.make_inputs(wl)
    beta, level = W.topology(wl)
    c_hat, pen, cap = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor,
                                           args.cap_mode)

    def up(a):
        t = torch.from_numpy(a)
        if wl.dtype == W.BF16:
            t = t.view(torch.int16).view(torch.bfloat16)
        return t.to(dev)

    x, w = up(inp["x"]), up(inp["w"])
    del inp
    S, d, N, P, k = wl.S, wl.d, wl.N, wl.P, wl.k
    b = wl.elem_bytes
    pen_d = torch.from_numpy(pen).to(dev)
    cap_d = torch.from_numpy(cap).to(dev)
    ws = T.workspace(S, d, N, P, k, wl.dtype, dev)
    i32, f32 = torch.int32, torch.float32
    topk_idx = torch.empty((S, k), dtype=i32, device=dev)
    topk_w = torch.empty((S, k), dtype=f32, device=dev)
    m = torch.empty((N,), dtype=f32, device=dev)
    c_expert = torch.empty((N,), dtype=i32, device=dev)
    c_device = torch.empty((P,), dtype=i32, device=dev)
    loss = torch.empty((1,), dtype=f32, device=dev)
    send = torch.empty((S * k, d), dtype=x.dtype, device=dev)
    slot = torch.empty((S, k), dtype=i32, device=dev)
    kept = torch.empty((N,), dtype=i32, device=dev)
    off = torch.empty((N + 1,), dtype=i32, device=dev)
    scd = torch.empty((P,), dtype=i32, device=dev)
    y = torch.empty((S, d), dtype=x.dtype, device=dev)
    stream = torch.cuda.current_stream()
    rotate = max(1, args.rotate)
    sets = [(x, send, y)] + [(x.clone(), torch.empty_like(send), torch.empty_like(y)) for _ in range(rotate - 1)]
    turn = [0]

    def step():
        xs, sends, ys = sets[turn[0] % rotate]
        turn[0] += 1
        # stream=None: the binding passes torch's current stream (the capture stream under --graph)
        T.tamoe_gate(xs, w, P, k, None, topk_idx, topk_w, m, c_expert, c_device, ws, None)
        T.tamoe_aux_loss(m, c_expert, pen_d, P, S, loss, None)
        T.tamoe_dispatch(xs, topk_idx, cap_d, N, P, sends, slot, kept, off, scd, ws, None)
        # identity expert: the rows come back as they were sent; S*k bounds the row count
        T.tamoe_combine(sends, S * k, slot, topk_w, ys, None)

    for _ in range(max(args.warmup, 0)):
        step()
    torch.cuda.synchronize()

    # yardstick, outside the timed region: a plain copy of x into y (same size)
    T.tamoe_trace_start(16)
    for _ in range(5):
        T.tamoe_copy_probe(x, y, stream)
    n_rec = T.tamoe_trace_stop()
    copy_us = float(np.median([T.tamoe_trace_get(i)[1] for i in range(n_rec)])) * 1e3
    copy_gbs = 2.0 * S * d * b / (copy_us * 1e-6) / 1e9

    # row-mix yardsticks on the realised slot table (k = 2, rows a multiple of 1 KiB): the scatter's
    # and the combine's memory operations with nothing else around them
    mix = None
    if k == 2 and (d * b) % 1024 == 0:
        r0 = slot[:, 0].contiguous()
        r1 = slot[:, 1].contiguous()
        T.tamoe_trace_start(16)
        for _ in range(5):
            T.tamoe_mix_probe(x, send, r0, r1, 1, None)
        n_rec = T.tamoe_trace_stop()
        sc_us = float(np.median([T.tamoe_trace_get(i)[1] for i in range(n_rec)])) * 1e3
        T.tamoe_trace_start(16)
        for _ in range(5):
            T.tamoe_mix_probe(send, y, r0, r1, 2, None)
        n_rec = T.tamoe_trace_stop()
        ga_us = float(np.median([T.tamoe_trace_get(i)[1] for i in range(n_rec)])) * 1e3
        K0 = int((slot >= 0).sum().item())
        live0 = int((slot >= 0).any(dim=1).sum().item())
        mix = {"scatter_1r2w": {"median_us": round(sc_us, 2),
                                "GBs": round((live0 + K0) * d * b / (sc_us * 1e-6) / 1e9, 1)},
               "gather_2r1w": {"median_us": round(ga_us, 2),
                               "GBs": round((K0 + S) * d * b / (ga_us * 1e-6) / 1e9, 1)}}

    launches_per_step = 9

    def collect():
        n = T.tamoe_trace_stop()
        out = {}
        for i in range(n):
            name, ms = T.tamoe_trace_get(i)
            out.setdefault(name, []).append(ms)
        return out

    # Pass 1 (not timed): every launch bracketed by HIP events -> the per-kernel table and the name
    # of the longest-running kernel.  Two event records per launch cost ~3 us of GPU time each, so
    # this pass is kept out of `value`.
    table_steps = max(1, min(args.steps, 20))
    T.tamoe_trace_filter(None)
    T.tamoe_trace_start(launches_per_step * table_steps)
    for _ in range(table_steps):
        step()
    torch.cuda.synchronize()
    per_kernel = collect()
    dominant = max(per_kernel, key=lambda n: float(np.mean(per_kernel[n])))

    run_step = step
    if args.graph:
        # the library only enqueues kernels on the current stream, so a step can be captured as is
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()                               # with --rotate the replays reuse the captured set
        run_step = graph.replay
        for _ in range(2):
            run_step()
        torch.cuda.synchronize()

    # Pass 2, the timed region: K steps; only the dominant kernel is bracketed by events (two
    # records per step), which is what `roofline.achieved` is computed from.
    traced_in_timed_region = not (args.no_trace or args.graph)
    if traced_in_timed_region:
        T.tamoe_trace_filter(dominant)
        T.tamoe_trace_start(args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    dominant_live = collect().get(dominant) if traced_in_timed_region else None
    T.tamoe_trace_filter(None)
    T.tamoe_trace_clear()

    # The other capacity mode beside the headline one (uniform <-> proportional to the target pattern):
    # a short timed region of its own, same buffers; restored afterwards.
    other_mode = None
    if not args.graph:
        K_main = int(off[-1].item())
        _, _, cap_o = T.tamoe_topo_pattern(beta, level, wl.P, wl.N, wl.rank, wl.k, wl.S, wl.capacity_factor,
                                           1 - args.cap_mode)
        cap_keep = cap_d.clone()
        cap_d.copy_(torch.from_numpy(cap_o).to(dev))
        n_o = max(1, min(args.steps, 20))
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_o):
            step()
        torch.cuda.synchronize()
        el_o = time.perf_counter() - t0
        K_o = int(off[-1].item())
        other_mode = {"cap_mode": 1 - args.cap_mode, "steps": n_o, "ms_per_step": round(el_o * 1e3 / n_o, 4),
                      "value": round(S * n_o / el_o, 1), "unit": "tokens/s", "kept_rows_K": K_o,
                      "drop_rate": round(1.0 - K_o / (S * k), 4)}
        cap_d.copy_(cap_keep)
        for _ in range(rotate):                  # slot, send and the size outputs are those of the headline mode again
            step()
        torch.cuda.synchronize()
        assert int(off[-1].item()) == K_main

    # Backward kernels (the next row of the scope after the forward path): measured in a pass of
    # their own with events around every launch; they are not part of `value`.
    backward = None
    if not args.no_backward:
        K_now = int(off[-1].item())
        logits = torch.empty((S, N), dtype=f32, device=dev)
        T.tamoe_gate(x, w, P, k, logits, topk_idx, topk_w, m, c_expert, c_device, ws, None)
        dy = y                                   # any tensor of the shape of y serves as upstream gradient
        d_recv = torch.empty((max(K_now, 1), d), dtype=x.dtype, device=dev)
        d_w = torch.empty((S, k), dtype=f32, device=dev)
        d_logits = torch.empty((S, N), dtype=f32, device=dev)
        d_x = torch.empty((S, d), dtype=x.dtype, device=dev)

        def bwd():
            T.tamoe_combine_bwd(dy, send, K_now, slot, topk_w, d_recv, d_w, None)
            T.tamoe_gate_bwd(logits, topk_idx, d_w, pen_d, c_expert, 1.0, P, d_logits, None)
            T.tamoe_dispatch_bwd(d_recv, K_now, slot, d_x, None)

        for _ in range(3):
            bwd()
        torch.cuda.synchronize()
        reps = 10
        T.tamoe_trace_start(3 * reps)
        for _ in range(reps):
            bwd()
        torch.cuda.synchronize()
        rec = collect()
        T.tamoe_trace_clear()
        live_b = int((slot >= 0).any(dim=1).sum().item())
        rowb = d * b
        bwd_bytes = {"combine_bwd_kernel": S * rowb + 2 * K_now * rowb + S * k * 12,
                     "gate_bwd_kernel": 2 * S * N * 4 + S * k * 8,
                     "dispatch_bwd_kernel": K_now * rowb + S * rowb + S * k * 4}
        backward = []
        for name, ts in rec.items():
            us = float(np.mean(ts)) * 1e3
            gbs = bwd_bytes[name] / (us * 1e-6) / 1e9
            backward.append({"kernel": name, "avg_us": round(us, 2), "algo_bytes": int(bwd_bytes[name]),
                             "achieved_GBs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4)})
        del logits, d_recv, d_w, d_logits, d_x

    # Receive-side regrouping (next row of the scope): the K_now rows of `send` stand in for a receive
    # buffer with P source chunks x E local experts (E = 2 when the workload has one expert per device,
    # where regrouping is the identity), seeded Poisson segment sizes.  Untimed pass, not part of `value`.
    regroup = None
    if not args.no_backward:
        E_r = wl.E if wl.E > 1 else 2
        P_r = min(wl.P, 128 // E_r)
        rows_r = int(off[-1].item())
        if rows_r >= P_r * E_r:
            rng = np.random.Generator(np.random.Philox(key=[wl.seed, 11]))
            share = rng.poisson(64, size=(P_r, E_r)).astype(np.float64) + 1.0
            cnt = np.floor(share / share.sum() * rows_r).astype(np.int32)
            cnt[0, 0] += rows_r - int(cnt.sum())
            cnt_d = torch.from_numpy(cnt).to(dev)
            rin = send[:rows_r]
            rout = torch.empty_like(rin)
            for _ in range(2):
                T.tamoe_regroup(rin, cnt_d, True, rout, None, ws, None)
            torch.cuda.synchronize()
            T.tamoe_trace_filter("regroup_copy_kernel")
            T.tamoe_trace_start(10)
            for _ in range(10):
                T.tamoe_regroup(rin, cnt_d, True, rout, None, ws, None)
            torch.cuda.synchronize()
            rec = collect()
            T.tamoe_trace_filter(None)
            T.tamoe_trace_clear()
            us = float(np.mean(rec["regroup_copy_kernel"])) * 1e3
            rb = 2 * rows_r * d * b
            regroup = {"kernel": "regroup_copy_kernel", "P": P_r, "E": E_r, "rows": rows_r, "avg_us": round(us, 2),
                       "algo_bytes": int(rb), "achieved_GBs": round(rb / (us * 1e-6) / 1e9, 1),
                       "frac_of_hbm_peak": round(rb / (us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4)}
            del rout

    # Variants (a further row of the scope): the fixed-size zero-padded layout against the packed one
    # (bytes written and time of the row movers), and the weight renormalisation.  Untimed pass.
    variants = None
    if not args.no_backward:
        C = int(cap_d.max().item())
        pad_rows = N * C
        send_p = torch.empty((pad_rows, d), dtype=x.dtype, device=dev)
        slot_p = torch.empty_like(slot)
        kept_p = torch.empty_like(kept)
        w_n = torch.empty_like(topk_w)
        d_wn = torch.empty_like(topk_w)

        def var():
            T.tamoe_dispatch_padded(x, topk_idx, cap_d, N, P, C, send_p, slot_p, kept_p, ws, None)
            T.tamoe_renorm_topk(topk_w, w_n, None)
            T.tamoe_renorm_topk_bwd(topk_w, w_n, d_wn, None)

        for _ in range(2):
            var()
        torch.cuda.synchronize()
        reps = 10
        T.tamoe_trace_start(7 * reps)
        for _ in range(reps):
            var()
        torch.cuda.synchronize()
        rec = collect()
        T.tamoe_trace_clear()
        K_p = int(kept_p.sum().item())
        live_p = int((slot_p >= 0).any(dim=1).sum().item())
        us = {n: float(np.mean(ts)) * 1e3 for n, ts in rec.items()}
        mover_us = us["dispatch_copy_kernel"] + us["dispatch_pad_fill_kernel"]
        mover_bytes = (live_p + pad_rows) * d * b + S * k * 8
        variants = {
            "padded_dispatch": {"C": C, "rows_written": pad_rows, "rows_kept": K_p,
                                "copy_us": round(us["dispatch_copy_kernel"], 2),
                                "pad_fill_us": round(us["dispatch_pad_fill_kernel"], 2),
                                "algo_bytes": int(mover_bytes),
                                "achieved_GBs": round(mover_bytes / (mover_us * 1e-6) / 1e9, 1),
                                "rows_vs_packed": round(pad_rows / max(K_p, 1), 4)},
            "renorm_topk_us": round(us["renorm_topk_kernel"], 2),
            "renorm_topk_bwd_us": round(us["renorm_topk_bwd_kernel"], 2),
        }
        del send_p, slot_p, kept_p, w_n, d_wn

    ms_per_step = elapsed * 1e3 / args.steps
    tokens_per_s = S * args.steps / elapsed

    # realised routing (for the algorithmic byte counts)
    K = int(off[-1].item())
    live_tokens = int((slot >= 0).any(dim=1).sum().item())
    row = d * b
    algo_bytes = {
        "gate_bf16_kernel": S * row + N * row + S * k * 8,
        "gate_gemm_f32_kernel": S * row + N * row + S * N * 4,
        "select_kernel": S * N * 4 + S * k * 8,
        "dispatch_copy_kernel": live_tokens * row + K * row + S * k * 8,
        "combine_kernel": K * row + S * row + S * k * 8,
    }
    kernels = []
    for name, ts in per_kernel.items():
        avg_ms = float(np.mean(ts))
        entry = {"kernel": name, "launches": len(ts), "avg_us": round(avg_ms * 1e3, 2)}
        if name in algo_bytes:
            entry["algo_bytes"] = int(algo_bytes[name])
            entry["achieved_GBs"] = round(algo_bytes[name] / (avg_ms * 1e-3) / 1e9, 1)
            entry["frac_of_hbm_peak"] = round(entry["achieved_GBs"] / HBM_PEAK_GBS, 4)
        kernels.append(entry)
    kernels.sort(key=lambda e: -e["avg_us"])
    roofline = None
    if dominant in algo_bytes:
        live = dominant_live if dominant_live else per_kernel[dominant]
        dom_us = float(np.mean(live)) * 1e3
        gbs = algo_bytes[dominant] / (dom_us * 1e-6) / 1e9
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                    "traffic": measured_traffic(wl.name, dominant),
                    "algo_bytes_per_launch": int(algo_bytes[dominant]), "avg_launch_us": round(dom_us, 2),
                    "launches_timed": len(live),
                    "timed_in": "timed region" if dominant_live else "table pass"}

    total_algo = algo_bytes["gate_bf16_kernel" if wl.dtype == W.BF16 else "gate_gemm_f32_kernel"] \
        + algo_bytes["dispatch_copy_kernel"] + algo_bytes["combine_kernel"]
    result = {
        "metric": "routed tokens/sec (gate+aux_loss+dispatch+combine), 1 GPU",
        "value": round(tokens_per_s, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == W.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": wl.name, "S": S, "d": d, "N": N, "k": k, "P": P, "E": wl.E,
                   "capacity_factor": wl.capacity_factor, "cap_mode": args.cap_mode,
                   "topology": f"{wl.nodes}x{wl.devs_per_node} ratio {wl.bw_ratio:g}:1", "rank": wl.rank,
                   "kept_rows_K": K, "tokens_with_a_kept_choice": live_tokens,
                   "drop_rate": round(1.0 - K / (S * k), 4), "rotating_buffer_sets": rotate},
        "path_algo_bytes_per_step": int(total_algo),
        "path_achieved_GBs": round(total_algo / (ms_per_step * 1e-3) / 1e9, 1),
        "roofline": roofline,
        "copy_probe": {"bytes_moved": int(2 * S * d * b), "median_us": round(copy_us, 2),
                       "GBs": round(copy_gbs, 1), "frac_of_hbm_peak": round(copy_gbs / HBM_PEAK_GBS, 4)},
        "mix_probe": mix,
        "kernels": kernels,
        "backward_kernels": backward,
        "regroup_kernel": regroup,
        "variants": variants,
        "other_capacity_mode": other_mode,
        "l_topo": float(loss.item()),
        "mode": "graph replay" if args.graph else "eager",
        "kernels_table_from": f"untimed pass of {table_steps} steps with HIP events around every launch",
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, W, args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
