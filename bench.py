#!/usr/bin/env python3
"""Benchmark of the HAG aggregation hot path on one MI355X.

A step = one hag_forward + one hag_backward (all phases: aggregation-node levels,
final gather; transposed levels, source gather) over one synthetic graph whose
feature matrices already live in HBM.  The default workload is benchmark config 3,
the largest one (degree-corrected SBM, 232,965 nodes, 114M directed edges, D=128,
capacity |V|/4, sum); configs 1, 2 and 4 ride along as short extra measurements.

Prints ONE JSON line (stdout); a human-readable breakdown goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E, published
# Limits derived from the chip's unit counts and clock (8 XCDs, 256 compute units, 2.4 GHz):
#   L2 -> compute units: 16 channels x 128 B/clk per XCD; the vector L1s take 64 B/clk per
#   compute unit, which is the same 39.3 TB/s;  LDS: 64 banks x 4 B per clock and compute unit.
L2_PEAK_GBS = 8 * 16 * 128 * 2.4
LDS_PEAK_GBS = 256 * 64 * 4 * 2.4

# L2 fills + write-backs per launch of the dominant kernel, from separate rocprofv3 --pmc runs of this
# file (FETCH_SIZE, WRITE_SIZE, scaled by what the same counters read for --copy-calibration's
# known copy); the summaries are in profiles/.  Not measured by the run that prints them.
PROFILED_TRAFFIC = {
    ("config2:holme_kim56944", 128, "sum"): dict(fetch=310725 * 2048, write=28472 * 1024,
                                                  source="profiles/pmc_config2_holme_kim56944_d128_sum.txt"),
    ("config3:dcsbm232965", 128, "sum"): dict(fetch=6014900 * 2048, write=931865 * 1024,
                                               source="profiles/pmc_config3_dcsbm232965_d128_sum.txt"),
    ("config4:er_batch5000x74", 64, "sum"): dict(fetch=74111 * 2048, write=92500 * 1024,
                                                  source="profiles/pmc_config4_er_batch5000x74_d64_sum.txt"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_workload(cfg: int, capacity, workloads, synth, device_search=False):
    t0 = time.time()
    rowptr, col, graph_ptr = synth.graph_for_config(cfg)
    log(f"[bench] config {cfg}: graph generated in {time.time() - t0:.1f}s")
    h = workloads.build_hag(cfg, rowptr, col, graph_ptr, capacity, log=lambda m: log("[bench] " + m),
                            device_search=device_search)
    return rowptr, col, h, workloads.FEATURE_DIM[cfg]


def time_steps(torch, fn, steps, warmup):
    """(median, mean) duration of `fn` in ms: `steps` timed repetitions after `warmup` untimed ones, every
    repetition bracketed by events on the launch stream; the mean is wall clock over the whole timed region."""
    for _ in range(warmup):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / steps * 1e3
    return statistics.median(a.elapsed_time(b) for a, b in ev), wall


def time_interleaved(torch, fn_a, fn_b, steps, warmup, blocks=4):
    """Per-step event times of two paths measured alternately: after `warmup` untimed steps of each, `steps`
    timed steps of each in `blocks` alternating runs (a, b, a, b, ...), so that a slow drift of the machine (clocks,
    what else shares it) lands on both.  Returns ((median_a, wall_mean_a), (median_b, wall_mean_b)) in ms."""
    for _ in range(warmup):
        fn_a()
    for _ in range(warmup):
        fn_b()
    per = [steps // blocks + (1 if i < steps % blocks else 0) for i in range(blocks)]
    samples, wall = ([], []), [0.0, 0.0]
    for n_block in per:
        for which, fn in ((0, fn_a), (1, fn_b)):
            fn()                                   # one untimed step after the switch of paths
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_block)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for a, b in ev:
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            wall[which] += time.perf_counter() - t0
            samples[which].extend(a.elapsed_time(b) for a, b in ev)
    return tuple((statistics.median(samples[w]), wall[w] / steps * 1e3) for w in (0, 1))


def time_kernel(torch, pre, fn, post, steps, warmup):
    """Median duration (ms) of `fn` inside the full step, bracketed by events on the launch stream."""
    for _ in range(warmup):
        pre(); fn(); post()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    for a, b in ev:
        pre()
        a.record()
        fn()
        b.record()
        post()
    torch.cuda.synchronize()
    return statistics.median(a.elapsed_time(b) for a, b in ev)


def measure_ceilings(torch, binding, d):
    """What this machine delivers for rows of d fp32 features read at random by sub-groups of lanes (the
    gather kernel's access shape, hag_probe_rows), by the level that serves them, and for a plain copy."""
    out = {}
    wgs = 256 * 16
    sink = torch.empty(wgs * 1024, dtype=torch.float32, device="cuda")
    d = min(d, 256)

    def rate(n_rows, reads, lds):
        src = torch.empty(n_rows * d, dtype=torch.float32, device="cuda").normal_()
        nbytes = 0
        for _ in range(2):
            nbytes = binding.probe_rows(src, n_rows, d, reads, lds, wgs, sink)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 5
        a.record()
        for _ in range(reps):
            binding.probe_rows(src, n_rows, d, reads, lds, wgs, sink)
        b.record()
        torch.cuda.synchronize()
        return nbytes * reps / (a.elapsed_time(b) * 1e-3) / 1e9

    def pow2_rows(nbytes):
        r = 1
        while r * 2 * d * 4 <= nbytes:
            r *= 2
        return r

    out["l2_resident_rows_GBps"] = rate(pow2_rows(2 << 20), 512, 0)        # 2 MB: every XCD's L2 holds all of it
    out["infinity_cache_rows_GBps"] = rate(pow2_rows(128 << 20), 256, 0)   # 128 MB: misses L2, fits the 256 MB memory-side cache
    out["hbm_rows_GBps"] = rate(pow2_rows(4 << 30), 128, 0)                # 4 GB: served by HBM
    out["lds_rows_GBps"] = rate(pow2_rows(1 << 20), 2048, 1)
    # what a row accumulator kept in LDS would cost: a row added into an LDS row by read-add-write, by LDS atomics
    out["lds_row_accumulate_GBps"] = rate(pow2_rows(1 << 20), 2048, 2)
    out["lds_row_atomic_add_GBps"] = rate(pow2_rows(1 << 20), 128, 3)
    n = 1 << 30
    src = torch.empty(n // 4, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    for _ in range(2):
        binding.probe_copy(src, dst, n)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        binding.probe_copy(src, dst, n)
    b.record()
    torch.cuda.synchronize()
    out["copy_1GiB_read_plus_write_GBps"] = 2.0 * n * 10 / (a.elapsed_time(b) * 1e-3) / 1e9
    out["row_width"] = d
    del src, dst, sink
    torch.cuda.empty_cache()
    return out


def cpu_baseline(oracle, synth, rowptr, col, h, d, seed, budget_s=24.0):
    """The oracle (fp64 accumulation) on the host, on a bounded sample: the whole graph and HAG, a slice of the
    feature columns.  Four legs: naive aggregation and Algorithm 2 over the HAG, each forward + backward, each
    on one thread and on all host threads the oracle's OpenMP loops use."""
    import ctypes

    import numpy as np

    st = h.stats()
    n = st["n"]
    f = h.get_forward()
    oh = oracle.Hag(n, f["agg_left"], f["agg_right"], f["hrowptr"], f["hcol"])
    deg = np.diff(rowptr)
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    gomp = ctypes.CDLL("libgomp.so.1")

    def leg(fn, nthreads, share):
        # columns sized so that one repetition takes roughly share seconds at ~1.5e8 elements/s/thread
        d_s = d
        while d_s > 1 and 2.0 * st["e"] * d_s / (1.5e8 * nthreads) > share:
            d_s //= 2
        x = synth.features_f32(n, d_s, seed)
        gy = synth.features_f32(n, d_s, seed + 1)
        gomp.omp_set_num_threads(nthreads)
        t0 = time.perf_counter()
        reps = 0
        while True:
            fn(x, gy)
            reps += 1
            if time.perf_counter() - t0 > share or reps >= 50:
                break
        dt = (time.perf_counter() - t0) / reps
        return {"feature_elems_per_s": 2.0 * st["e"] * d_s / dt, "threads": nthreads, "columns": d_s, "reps": reps}

    def naive(x, gy):
        oracle.naive_forward(rowptr, col, x, "sum")
        oracle.naive_backward(rowptr, col, gy, "sum")

    def hag(x, gy):
        oracle.hag_forward(oh, deg, x, "sum")
        oracle.hag_backward(oh, deg, gy, "sum")

    share = budget_s / 4
    legs = {"hag_all_threads": leg(hag, threads, share), "naive_all_threads": leg(naive, threads, share),
            "hag_1_thread": leg(hag, 1, share), "naive_1_thread": leg(naive, 1, share)}
    gomp.omp_set_num_threads(threads)
    main = legs["hag_all_threads"]
    return {
        "value": main["feature_elems_per_s"],
        "unit": "feature-elems/s",
        "cores": threads,
        "kind": "oracle",
        "sample": f"Algorithm 2 over the whole graph and HAG, forward+backward, {main['columns']} of {d} feature columns, "
                  f"{main['reps']} reps; fp64 accumulation; OpenMP only on the oracle's loops with independent "
                  f"iterations, the rest serial",
        "legs": legs,
    }


def gcn_epoch_ms(torch, h, x, hidden, classes, steps, warmup, naive):
    """Per-epoch time (forward + backward) of a 2-layer GCN with `hidden` hidden dims and a SoftMax
    loss, the model of the paper's end-to-end measurement (Section 5.3), on the synthetic graph
    (paper_1906_03707_amd.layers.gcn2_loss: dense parts torch, aggregation hag_forward / hag_backward
    with op "gcn", or the naive-CSR baseline)."""
    from paper_1906_03707_amd import layers

    n, d = x.shape
    gen = torch.Generator(device="cuda").manual_seed(1)
    w1 = (torch.randn(d, hidden, device="cuda", generator=gen) / d ** 0.5).requires_grad_()
    w2 = (torch.randn(hidden, classes, device="cuda", generator=gen) / hidden ** 0.5).requires_grad_()
    labels = torch.randint(0, classes, (n,), device="cuda", generator=gen)

    def epoch():
        loss = layers.gcn2_loss(h, x, w1, w2, labels, naive=naive)
        w1.grad = w2.grad = None
        loss.backward()

    return time_steps(torch, epoch, steps, warmup)[0]


def sage_pool_epoch_ms(torch, h, x, hidden, classes, steps, warmup, naive):
    """Per-epoch time (forward + backward) of a 2-layer GraphSAGE with the pooling aggregator of
    Table 1 (paper_1906_03707_amd.layers.sage_pool2_loss: dense parts torch; the element-wise max,
    argmax kept for the backward pass, is hag_forward / hag_backward with op "max", or the baseline)."""
    from paper_1906_03707_amd import layers

    n, d = x.shape
    gen = torch.Generator(device="cuda").manual_seed(2)
    dims = [d, hidden, classes]
    pool = [(torch.randn(dims[i], hidden, device="cuda", generator=gen) / dims[i] ** 0.5).requires_grad_() for i in range(2)]
    comb = [(torch.randn(hidden + dims[i], dims[i + 1], device="cuda", generator=gen) / (hidden + dims[i]) ** 0.5).requires_grad_()
            for i in range(2)]
    labels = torch.randint(0, classes, (n,), device="cuda", generator=gen)

    def epoch():
        loss = layers.sage_pool2_loss(h, x, pool, comb, labels, naive=naive)
        for w in pool + comb:
            w.grad = None
        loss.backward()

    return time_steps(torch, epoch, steps, warmup)[0]


def sweep_config5(torch, synth, workloads, steps, warmup):
    """benchmark config 5: the 232,965-node graph over capacity {0, |V|/8, |V|/4, |V|/2} x feature
    dim {16, 128, 512} x {max, sum}, forward + backward.  One JSON line per point on stdout."""
    rowptr, col, _ = synth.graph_for_config(5)
    n = rowptr.size - 1
    log(f"[bench] config 5 sweep: graph ready ({col.size} directed edges)")
    hags = {}
    for cap in (0, n // 8, n // 4, n // 2):
        hags[cap] = workloads.build_hag(5, rowptr, col, None, cap, log=lambda m: log("[bench] " + m)).upload()
    log("[bench] capacity      d  op    hag ms   naive ms  speedup  aggregations fewer")
    for d in (16, 128, 512):
        x = torch.from_numpy(synth.features_f32(n, d, synth.SEED_BASE + 5 + 1000 + d)).cuda()
        gy = torch.from_numpy(synth.features_f32(n, d, synth.SEED_BASE + 5 + 2000 + d)).cuda()
        y, gx = torch.empty_like(x), torch.empty_like(x)
        am = torch.empty((n, d), dtype=torch.int32, device="cuda")
        for op in ("max", "sum"):
            for cap, h in hags.items():
                st = h.stats()
                a = am if op == "max" else None

                def step_hag():
                    h.forward(x, op, y=y, argmax=a)
                    h.backward(gy, op, argmax=a, gx=gx)

                def step_naive():
                    h.naive_forward(x, op, y=y, argmax=a)
                    h.naive_backward(gy, op, argmax=a, gx=gx)

                (ms_h, _), (ms_n, _) = time_interleaved(torch, step_hag, step_naive, steps, warmup, blocks=2)
                red = st["aggr_naive"] / max(st["aggr_hag"], 1)
                log(f"[bench] {cap:8d} {d:6d}  {op:4s} {ms_h:8.3f}  {ms_n:8.3f}  {ms_n / ms_h:6.3f}x  {red:6.3f}x")
                print(json.dumps({"workload": "config5:dcsbm232965_sweep", "capacity": cap, "feature_dim": d, "op": op,
                                  "ms_per_step": ms_h, "naive_ms_per_step": ms_n, "speedup_vs_naive": ms_n / ms_h,
                                  "value": 2.0 * st["e"] * d / (ms_h * 1e-3), "unit": "feature-elems/s",
                                  "aggregation_reduction": red, "levels": st["levels"], "stages": st["stages"]}),
                      flush=True)
        del x, gy, y, gx, am
        torch.cuda.empty_cache()


FP32_MFMA_PEAK_TFLOPS = 157.3


def seq_lstm_bench(torch, binding, synth, cfg, first_k, d, hidden, steps, warmup, only=None):
    """LSTM aggregator over ordered neighbour lists (Section 3.1's sequential Aggregate): every node's list is its
    first `first_k` neighbours in ascending id order; the plain lists against prefix HAGs of capacity |V|/4 and
    unlimited.  One step = one forward pass (all cell evaluations of the plan)."""
    import numpy as np
    rowptr, col, _ = synth.graph_for_config(cfg)
    n = rowptr.size - 1
    from paper_1906_03707_amd import workloads
    rp, cl = workloads.first_neighbour_lists(rowptr, col, first_k)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    x, w_ih, w_hh, b = (dev(a) for a in workloads.lstm_inputs(cfg, n, d, hidden))
    out = torch.empty((n, hidden), dtype=torch.float32, device="cuda")
    capacities = {"lists": 0, "hag_quarter": n // 4, "hag_unlimited": int(cl.size)}
    # `only` (one plan's name): that plan alone, nothing interleaved -- for counter runs, where every launch of the kernel
    # should be the same work
    plans = {name: binding.SeqHag(rp, cl, cap).upload() for name, cap in capacities.items() if only in (None, name)}
    # what the matrix cores deliver on this machine for the instruction the kernel uses
    sink = torch.empty(256 * 8 * 256, dtype=torch.float32, device="cuda")
    binding.probe_mfma_f32(2000, 256 * 8, sink)
    ea, eb = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ea.record()
    probe_flops = sum(binding.probe_mfma_f32(20000, 256 * 8, sink) for _ in range(3))
    eb.record()
    torch.cuda.synchronize()
    mfma_ceiling = probe_flops / (ea.elapsed_time(eb) * 1e-3) / 1e12
    log(f"[bench] fp32 matrix-core probe: {mfma_ceiling:.1f} TFLOP/s (published peak {FP32_MFMA_PEAK_TFLOPS})")
    flops_per_cell = 2.0 * 4 * hidden * (d + hidden)
    res = {"workload": f"config{cfg}:{synth.CONFIGS[cfg]['name']}, first {first_k} neighbours in id order", "nodes": n,
           "list_entries": int(cl.size), "d": d, "hidden": hidden, "flops_per_cell": flops_per_cell,
           "measured_fp32_matrix_TFLOPs": mfma_ceiling, "plans": {}}
    base = (lambda: plans["lists"].lstm_forward(x, w_ih, w_hh, b, out=out)) if "lists" in plans else None
    for name, p in plans.items():
        fn = (lambda p=p: p.lstm_forward(x, w_ih, w_hh, b, out=out))
        if name == "lists" or base is None:
            ms, _ = time_steps(torch, fn, steps, warmup)
            ms_base = ms if name == "lists" else float("nan")
        else:
            (ms, _), (ms_base, _) = time_interleaved(torch, fn, base, steps, warmup)
        tf = p.cells * flops_per_cell / (ms * 1e-3) / 1e12
        res["plans"][name] = {"cells": p.cells, "aggregation_nodes": p.merges, "launches": p.launches, "levels": int(p.plan()[4].size - 1), "longest_chain": p.ranks, "ms_per_pass": ms,
                              "lists_ms_per_pass": ms_base, "speedup_vs_lists": ms_base / ms,
                              "cells_fewer": int(cl.size) / max(p.cells, 1), "tflops": tf,
                              "frac_of_fp32_matrix_peak": tf / FP32_MFMA_PEAK_TFLOPS, "frac_of_measured_ceiling": tf / mfma_ceiling}
        log(f"[bench] LSTM aggregator, {name}: {p.cells} cells ({res['plans'][name]['cells_fewer']:.2f}x fewer), {p.launches} launches, "
            f"{ms:.3f} ms per pass ({ms_base / ms:.2f}x the plain lists' speed), {tf:.1f} TFLOP/s = "
            f"{100 * tf / FP32_MFMA_PEAK_TFLOPS:.1f}% of the fp32 matrix-core peak")
    # training: forward keeping the tape + backward (gradients of x and of the LSTM's parameters), where the sizes allow
    if plans and next(iter(plans.values())).train_workspace_bytes(d, hidden) > 0:
        g_a = torch.from_numpy(np.random.default_rng(synth.SEED_BASE + 100 * cfg + 8).normal(size=(n, hidden)).astype(np.float32)).cuda()
        ws = torch.empty(max(p.train_workspace_bytes(d, hidden) for p in plans.values()), dtype=torch.uint8, device="cuda")
        def train_step(p):
            p.lstm_forward_train(x, w_ih, w_hh, b, workspace=ws)
            p.lstm_backward(x, w_ih, w_hh, g_a, ws)
        for name, p in plans.items():
            ms, _ = time_steps(torch, lambda p=p: train_step(p), steps, warmup)
            p.lstm_forward_train(x, w_ih, w_hh, b, workspace=ws)
            ms_f, _ = time_steps(torch, lambda p=p: p.lstm_forward_train(x, w_ih, w_hh, b, workspace=ws), steps, warmup)
            res["plans"][name]["train_step_ms"] = ms
            res["plans"][name]["forward_train_ms"] = ms_f
            res["plans"][name]["train_workspace_GB"] = p.train_workspace_bytes(d, hidden) / 1e9
        base_ms = res["plans"]["lists"]["train_step_ms"] if "lists" in plans else float("nan")
        for name in plans:
            r = res["plans"][name]
            r["train_step_speedup_vs_lists"] = base_ms / r["train_step_ms"]
            r["train_step_tflops"] = 3 * r["cells"] * flops_per_cell / (r["train_step_ms"] * 1e-3) / 1e12
            log(f"[bench] LSTM aggregator training step (forward + backward), {name}: {r['train_step_ms']:.3f} ms "
                f"(forward {r['forward_train_ms']:.3f}; {r['train_step_speedup_vs_lists']:.2f}x the plain lists' speed; "
                f"{r['train_step_tflops']:.1f} TFLOP/s over 3x the forward flops; workspace {r['train_workspace_GB']:.1f} GB)")
        del ws
    # inference latency of a 2-layer GraphSAGE with LSTM aggregators around the same passes (Section 5.3 reports inference
    # latency next to training time); dense Update in torch, `hidden` wide throughout, 16 classes
    from paper_1906_03707_amd import layers
    gen = torch.Generator(device="cuda").manual_seed(3)
    dims = [d, hidden, 16]
    cells = [(torch.randn(4 * hidden, dims[i], device="cuda", generator=gen) * 0.3, torch.randn(4 * hidden, hidden, device="cuda", generator=gen) * 0.3,
              torch.randn(4 * hidden, device="cuda", generator=gen) * 0.3) for i in range(2)]
    comb = [torch.randn(hidden + dims[i], dims[i + 1], device="cuda", generator=gen) / (hidden + dims[i]) ** 0.5 for i in range(2)]
    infer = {name: (lambda p=p: layers.sage_lstm2_logits(p, x, cells, comb)) for name, p in plans.items()}
    for name, fn in infer.items():
        if name == "lists" or "lists" not in infer:
            ms, _ = time_steps(torch, fn, steps, warmup)
            ms_base = ms if name == "lists" else float("nan")
        else:
            (ms, _), (ms_base, _) = time_interleaved(torch, fn, infer["lists"], steps, warmup)
        res["plans"][name]["sage_lstm2_inference_ms"] = ms
        res["plans"][name]["sage_lstm2_inference_speedup_vs_lists"] = ms_base / ms
        log(f"[bench] 2-layer GraphSAGE-LSTM inference, {name}: {ms:.3f} ms ({ms_base / ms:.2f}x the plain lists' speed)")
    # and its training epoch (forward + backward through both layers; Section 5.3's other figure), where the sizes allow
    if plans and next(iter(plans.values())).train_workspace_bytes(d, hidden) > 0:
        labels = torch.randint(0, 16, (n,), device="cuda", generator=gen)
        params = [t.requires_grad_() for c in cells for t in c] + [w.requires_grad_() for w in comb]
        def epoch(p):
            for t in params:
                t.grad = None
            layers.sage_lstm2_loss(p, x, cells, comb, labels).backward()
        base_ms = None
        for name, p in plans.items():
            ms, _ = time_steps(torch, lambda p=p: epoch(p), max(steps // 2, 3), 2)
            base_ms = ms if name == "lists" else base_ms
            res["plans"][name]["sage_lstm2_epoch_ms"] = ms
            res["plans"][name]["sage_lstm2_epoch_speedup_vs_lists"] = (base_ms / ms) if base_ms else float("nan")
            log(f"[bench] 2-layer GraphSAGE-LSTM training epoch, {name}: {ms:.3f} ms"
                + (f" ({base_ms / ms:.2f}x the plain lists' speed)" if base_ms else ""))
    return res


def short_workload(torch, binding, synth, workloads, cfg, steps, warmup):
    """Forward + backward of one of the smaller configs, HAG against the naive-CSR kernels: the figures
    that ride along with the main workload's line."""
    rowptr, col, h, d = build_workload(cfg, None, workloads, synth)
    st = h.stats()
    n = st["n"]
    h.upload()
    seed = synth.SEED_BASE + cfg
    x = torch.from_numpy(synth.features_f32(n, d, seed + 1000)).cuda()
    gy = torch.from_numpy(synth.features_f32(n, d, seed + 2000)).cuda()
    y, gx = torch.empty_like(x), torch.empty_like(x)

    def step_hag():
        h.forward(x, "sum", y=y)
        h.backward(gy, "sum", gx=gx)

    def step_naive():
        h.naive_forward(x, "sum", y=y)
        h.naive_backward(gy, "sum", gx=gx)

    (ms_h, _), (ms_n, _) = time_interleaved(torch, step_hag, step_naive, steps, warmup)
    red = st["aggr_naive"] / max(st["aggr_hag"], 1)
    log(f"[bench] config {cfg} (d={d}, sum): hag {ms_h:.4f} ms  naive {ms_n:.4f} ms  speedup {ms_n / ms_h:.3f}x  "
        f"(aggregations {red:.3f}x fewer)")
    return {"feature_dim": d, "nodes": n, "edges": st["e"], "capacity": st["a"], "ms_per_step": ms_h,
            "naive_ms_per_step": ms_n, "speedup_vs_naive": ms_n / ms_h, "aggregation_reduction": red,
            "transfer_reduction": st["xfer_naive"] / max(st["xfer_hag"], 1),
            "feature_elems_per_s": 2.0 * st["e"] * d / (ms_h * 1e-3), "levels": st["levels"], "stages": st["stages"]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3,
                    help="benchmark config (1-based); 3, the largest single-GPU workload, is the headline; 5 runs the "
                         "capacity x width x op sweep")
    ap.add_argument("--op", default="sum", choices=["sum", "mean", "max", "gcn"])
    ap.add_argument("--d", type=int, default=0, help="override the feature dimension")
    ap.add_argument("--capacity", type=int, default=-1, help="override the HAG capacity (default |V|/4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of configs 1, 2 and 4")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the probe kernels that measure the machine's ceilings (profiler runs); the roofline then "
                         "carries the derived peak only")
    ap.add_argument("--device-search", action="store_true",
                    help="build the HAG with hag_search + HAG_SEARCH_DEVICE (pair counting on the GPU) instead of "
                         "the host search / the cached merge list; the search time is logged to stderr")
    ap.add_argument("--sage-epoch", action="store_true",
                    help="also time one epoch of a 2-layer GraphSAGE with the max-pooling aggregator (16 hidden dims)")
    ap.add_argument("--gcn-epoch", action="store_true",
                    help="also time a 2-layer GCN epoch (16 hidden dims, SoftMax) around the aggregation")
    ap.add_argument("--seq-lstm", action="store_true",
                    help="time the LSTM aggregator over ordered lists (first 16 neighbours of --config 4 or 2, d = hidden = --d or 64): "
                         "plain lists against prefix HAGs")
    ap.add_argument("--seq-plan", choices=["lists", "hag_quarter", "hag_unlimited"], default=None,
                    help="with --seq-lstm: time this plan alone (every launch of the kernel is then the same work: for counter runs)")
    ap.add_argument("--one-launch", action="store_true",
                    help="run the HAG passes with the one-launch schedule (all stages and the gather over V in a single "
                         "kernel launch; off by default because it measures slower)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (hag_probe_copy: known traffic) so that rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings of the same run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1")

    import numpy as np
    import torch

    from paper_1906_03707_amd import binding, synth, workloads

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible (the HIP path has no CPU fallback)")
    binding.lib()
    torch.cuda.set_device(0)
    cfg = args.config
    if args.seq_lstm:
        c = cfg if cfg in (1, 2, 4) else 4
        width = args.d if args.d else 64
        res = seq_lstm_bench(torch, binding, synth, c, 16, width, width, max(args.steps // 2, 5), 3, only=args.seq_plan)
        main_plan = res["plans"][args.seq_plan or "hag_quarter"]
        print(json.dumps({"metric": "LSTM aggregator over ordered lists, forward: cell evaluations/s", "unit": "cells/s",
                          "value": main_plan["cells"] / (main_plan["ms_per_pass"] * 1e-3),
                          "n_gpus": 1, "dtype": "f32", "data": "synthetic", "higher_is_better": True, "vs_baseline": None,
                          # the pass is one launch of the cell kernel: its flops over the pass's time (pack and output kernels included)
                          "roofline": {"bound": "mfma", "achieved": main_plan["tflops"], "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                                       "frac": main_plan["tflops"] / FP32_MFMA_PEAK_TFLOPS, "traffic": None},
                          "config": res}), flush=True)
        return
    if cfg == 5:
        sweep_config5(torch, synth, workloads, max(min(args.steps, 10), 3), 2)
        return
    rowptr, col, h, d = build_workload(cfg, None if args.capacity < 0 else args.capacity, workloads, synth,
                                       device_search=args.device_search)
    if args.d:
        d = args.d
    op = args.op
    st = h.stats()
    n, e = st["n"], st["e"]
    h.upload()
    if args.one_launch:
        h.set_option(binding.HAG_OPT_ONE_LAUNCH_MAX_ITEMS, 1 << 20)
    seed = synth.SEED_BASE + cfg
    x = torch.from_numpy(synth.features_f32(n, d, seed + 1000)).cuda()
    gy = torch.from_numpy(synth.features_f32(n, d, seed + 2000)).cuda()
    y = torch.empty_like(x)
    gx = torch.empty_like(x)
    am = torch.empty((n, d), dtype=torch.int32, device="cuda") if op == "max" else None

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        binding.probe_copy(a, b, 1 << 30)    # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b

    def step_hag():
        h.forward(x, op, y=y, argmax=am)
        h.backward(gy, op, argmax=am, gx=gx)

    def step_naive():
        h.naive_forward(x, op, y=y, argmax=am)
        h.naive_backward(gy, op, argmax=am, gx=gx)

    def time_cold(fn, reps=5):
        """One step right after a write sweep over 1 GiB (larger than L2 + the 256 MB Infinity Cache)."""
        flush = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        tot = 0.0
        for i in range(reps):
            flush.fill_(float(i))
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(); fn(); b.record()
            torch.cuda.synchronize()
            tot += a.elapsed_time(b)
        return tot / reps

    # the timed region: exactly `steps` steps after `warmup` untimed ones, in four runs that alternate with the
    # baseline's (the machine's clocks drift by a few per cent over seconds: both paths get the same share of it)
    (ms_hag, ms_hag_wall), (ms_naive, ms_naive_wall) = time_interleaved(torch, step_hag, step_naive, args.steps, args.warmup)
    (ms_fwd, _), (ms_nfwd, _) = time_interleaved(torch, lambda: h.forward(x, op, y=y, argmax=am),
                                                 lambda: h.naive_forward(x, op, y=y, argmax=am), args.steps, args.warmup)

    def capture(fn):
        """The same step captured once into a HIP graph (replayed without per-launch host work)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    g_hag, g_naive = capture(step_hag), capture(step_naive)
    (ms_hag_graph, _), (ms_naive_graph, _) = time_interleaved(torch, g_hag.replay, g_naive.replay, args.steps, args.warmup)
    del g_hag, g_naive
    ms_hag_cold = time_cold(step_hag)
    ms_naive_cold = time_cold(step_naive)

    # dominant kernel, timed inside the step: the final gather of hag_forward (one launch per step), or, for a
    # batch of small graphs, the one launch that is the whole forward pass and serves every row read from LDS
    P = binding
    row = 4 * d
    lpr = min(64, max(4, 1 << (max(d // 4, 1) - 1).bit_length()))
    component_pass = st.get("components", 0) > 0 and op != "max" and os.environ.get("HAG_COMPONENT", "1") != "0"
    if component_pass:
        ms_gather = time_kernel(torch, lambda: None, lambda: h.forward(x, op, y=y, argmax=am),
                                lambda: h.backward(gy, op, argmax=am, gx=gx), args.steps, args.warmup)
        gather_bytes = h.algorithmic_bytes(0, op, d)
        kernel_name = f"component_kernel<float, {lpr}, 256, 0>"   # the whole forward pass
    else:
        ms_gather = time_kernel(
            torch,
            lambda: h.forward_phases(x, P.HAG_PHASE_LEVELS, op, y=y, argmax=am),
            lambda: h.forward_phases(x, P.HAG_PHASE_GATHER, op, y=y, argmax=am),
            lambda: (h.forward_phases(x, P.HAG_PHASE_FOLD, op, y=y, argmax=am), h.backward(gy, op, argmax=am, gx=gx)),
            args.steps, args.warmup)
        gather_bytes = (row + 4) * st["h"] + (row + 16) * n   # row reads + index reads, row writes + schedule
        if op == "max":
            gather_bytes += row * n                           # argmax rows written beside the values
        kernel_name = f"gather_kernel<float, {1 if op == 'max' else 0}, {lpr}, 0>"
    achieved = gather_bytes / (ms_gather * 1e-3) / 1e9
    workload = f"config{cfg}:{synth.CONFIGS[cfg]['name']}"
    ceil = measure_ceilings(torch, binding, d) if not args.no_ceilings else None

    # Which limit binds.  Rows of a cache-resident matrix never reach HBM, so algorithmic bytes per second may
    # exceed the HBM peak: the gather is then priced against what the L2s can hand to the compute units (peak
    # derived from unit counts and clock; beside it what hag_probe_rows reaches on this machine), the
    # component pass against the LDS read rate.  The HBM-equivalent figure stays as a key of its own.
    def measured(key):
        return None if ceil is None else ceil[key]

    if component_pass:
        bound, peak, ceiling = "lds", LDS_PEAK_GBS, measured("lds_rows_GBps")
        # every list entry is one LDS row read; staging adds one LDS write per row of the matrix
        achieved_bound = (row * st["e_hag"] + row * (n + st["a"])) / (ms_gather * 1e-3) / 1e9
    elif achieved > HBM_PEAK_GBS * 0.6:
        bound, peak, ceiling = "l2", L2_PEAK_GBS, measured("l2_resident_rows_GBps")
        achieved_bound = achieved
    else:
        bound, peak, ceiling = "hbm", HBM_PEAK_GBS, measured("hbm_rows_GBps")
        achieved_bound = achieved
    prof = PROFILED_TRAFFIC.get((workload, d, op)) if args.capacity < 0 else None
    roofline = {"bound": bound, "achieved": achieved_bound, "peak": peak, "unit": "GB/s", "frac": achieved_bound / peak,
                "traffic": None if prof is None else prof["fetch"] + prof["write"],
                "kernel": kernel_name, "kernel_ms": ms_gather, "algorithmic_bytes": gather_bytes,
                "measured_ceiling": ceiling, "frac_of_measured_ceiling": None if ceiling is None else achieved_bound / ceiling,
                "hbm_equivalent_frac": achieved / HBM_PEAK_GBS}
    if prof is not None:
        roofline["traffic_source"] = prof["source"] + " (a separate rocprofv3 --pmc run, not this run)"
        # L2 fills of the launch against what random rows out of the memory-side cache reach on this machine
        roofline["l2_fill"] = {"bytes": prof["fetch"], "achieved": prof["fetch"] / (ms_gather * 1e-3) / 1e9, "unit": "GB/s",
                               "measured_ceiling": measured("infinity_cache_rows_GBps")}

    alg_hag = h.algorithmic_bytes(0, op, d) + h.algorithmic_bytes(1, op, d)
    alg_naive = h.algorithmic_bytes(2, op, d) + h.algorithmic_bytes(3, op, d)
    # what must move at least: every input row in, every output row out, aggregation rows out and in,
    # indices once (forward + backward)
    b_min = 2 * (row * (2 * n + 2 * st["a"]) + 4 * st["e_hag"] + 16 * (n + st["a"]))
    value = 2.0 * e * d / (ms_hag * 1e-3)
    out = {
        "metric": "HAG agg fwd+bwd: feature-elems/s, HBM GB/s (% peak), speedup vs naive CSR",
        "value": value,
        "unit": "feature-elems/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_hag,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": workload, "nodes": n, "edges": e, "feature_dim": d, "op": op,
                   "capacity": st["a"], "levels": st["levels"], "hag_edges": st["e_hag"]},
        "roofline": roofline,
        "timing": "median of per-step event pairs on the launch stream over the timed steps, taken in four runs that "
                  "alternate with the naive baseline's",
        "ms_per_step_wall_mean": ms_hag_wall,
        "effective_GBps_fwd_bwd": alg_hag / (ms_hag * 1e-3) / 1e9,
        "effective_frac_of_hbm_peak": alg_hag / (ms_hag * 1e-3) / 1e9 / HBM_PEAK_GBS,
        "compulsory_bytes_fwd_bwd": b_min,
        "profiled_bytes_per_aggregated_element": None if prof is None else (prof["fetch"] + prof["write"]) / (e * d),
        "naive_csr": {"ms_per_step": ms_naive, "ms_per_step_wall_mean": ms_naive_wall,
                      "feature_elems_per_s": 2.0 * e * d / (ms_naive * 1e-3),
                      "effective_GBps": alg_naive / (ms_naive * 1e-3) / 1e9},
        "speedup_vs_naive": ms_naive / ms_hag,
        "aggregation_reduction": st["aggr_naive"] / max(st["aggr_hag"], 1),
        "transfer_reduction": st["xfer_naive"] / max(st["xfer_hag"], 1),
        "forward_ms": {"hag": ms_fwd, "naive": ms_nfwd},
        "cold_cache_ms_per_step": {"hag": ms_hag_cold, "naive": ms_naive_cold},
        "hip_graph_replay_ms_per_step": {"hag": ms_hag_graph, "naive": ms_naive_graph},
        "ceilings_GBps": ceil,
        "one_launch_schedule": bool(args.one_launch),
    }
    log(f"[bench] {workload} D={d} op={op}: N={n} E={e} A={st['a']} levels={st['levels']} E^={st['e_hag']}")
    log(f"[bench] fwd+bwd  hag {ms_hag:.4f} ms  naive {ms_naive:.4f} ms  speedup {ms_naive / ms_hag:.3f}x "
        f"(aggregations {out['aggregation_reduction']:.3f}x, transfers {out['transfer_reduction']:.3f}x fewer)")
    log(f"[bench] fwd only hag {ms_fwd:.4f} ms  naive {ms_nfwd:.4f} ms")
    log(f"[bench] replayed from a HIP graph: hag {ms_hag_graph:.4f} ms  naive {ms_naive_graph:.4f} ms")
    log(f"[bench] cold caches (after a 1 GiB write sweep): hag {ms_hag_cold:.4f} ms  naive {ms_naive_cold:.4f} ms")
    if ceil is not None:
        log(f"[bench] ceilings (rows of {ceil['row_width']} floats, GB/s): L2-resident {ceil['l2_resident_rows_GBps']:.0f}  "
            f"memory-side cache {ceil['infinity_cache_rows_GBps']:.0f}  HBM {ceil['hbm_rows_GBps']:.0f}  LDS {ceil['lds_rows_GBps']:.0f}  "
            f"1 GiB copy {ceil['copy_1GiB_read_plus_write_GBps']:.0f}")
    log(f"[bench] effective (algorithmic) GB/s fwd+bwd: hag {out['effective_GBps_fwd_bwd']:.0f}  "
        f"naive {out['naive_csr']['effective_GBps']:.0f}  (HBM peak {HBM_PEAK_GBS:.0f})")
    log(f"[bench] dominant kernel {kernel_name}: {ms_gather * 1e3:.1f} us, {gather_bytes / 1e6:.1f} MB -> {achieved_bound:.0f} GB/s "
        f"= {100 * achieved_bound / peak:.1f}% of the {bound} limit ({peak:.0f})"
        + ("" if ceiling is None else f", {100 * achieved_bound / ceiling:.1f}% of the measured ceiling ({ceiling:.0f})"))
    if args.sage_epoch:
        e_hag = sage_pool_epoch_ms(torch, h, x, 16, 16, max(args.steps // 4, 5), 3, naive=False)
        e_naive = sage_pool_epoch_ms(torch, h, x, 16, 16, max(args.steps // 4, 5), 3, naive=True)
        out["sage_pool_epoch_ms"] = {"hag": e_hag, "naive": e_naive, "hidden": 16, "classes": 16, "layers": 2}
        log(f"[bench] 2-layer GraphSAGE-P epoch (hidden 16): hag {e_hag:.3f} ms  naive {e_naive:.3f} ms  ({e_naive / e_hag:.2f}x)")
    if args.gcn_epoch:
        e_hag = gcn_epoch_ms(torch, h, x, 16, 16, max(args.steps // 4, 5), 3, naive=False)
        e_naive = gcn_epoch_ms(torch, h, x, 16, 16, max(args.steps // 4, 5), 3, naive=True)
        out["gcn_epoch_ms"] = {"hag": e_hag, "naive": e_naive, "hidden": 16, "classes": 16, "layers": 2}
        log(f"[bench] 2-layer GCN epoch (16 hidden dims, SoftMax, fwd+bwd): hag {e_hag:.4f} ms  naive {e_naive:.4f} ms  "
            f"speedup {e_naive / e_hag:.3f}x")
    if not args.no_cpu_baseline:
        import oracle

        out["cpu_baseline"] = cpu_baseline(oracle, synth, rowptr, col, h, d, seed + 3000)
        cb = out["cpu_baseline"]
        log(f"[bench] cpu oracle, feature-elems/s: " + "  ".join(f"{k} {v['feature_elems_per_s']:.3e}" for k, v in cb["legs"].items())
            + f"  ({cb['cores']} threads)")
    del x, gy, y, gx, am, h
    torch.cuda.empty_cache()
    if cfg == 3 and not args.no_others and args.capacity < 0 and not args.d and op == "sum":
        out["other_workloads"] = {f"config{c}:{synth.CONFIGS[c]['name']}":
                                  short_workload(torch, binding, synth, workloads, c, 100, 10) for c in (1, 2, 4)}
        # the sequential Aggregate (LSTM over ordered lists): plain lists against prefix HAGs
        out["seq_lstm"] = seq_lstm_bench(torch, binding, synth, 4, 16, 64, 64, 20, 3)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
