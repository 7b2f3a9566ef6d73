#!/usr/bin/env python3
"""Throughput of the segment training step on one MI355X.

    python bench.py [--config 4] [--steps K] [--warmup W] [--no-cpu] [--no-e2e] [--no-others]

A "step" is one pass of the whole hot path -- forward, loss, backward confined to
the segment, SGD update -- of EVERY segment of the chosen configuration over one
batch of synthetic input that is already resident in HBM.  The default workload
is the comparison configuration (784-16384-16384-16384 | 16384-16384-16384-1000,
bf16 with float32 accumulation and master weights, batch 8192): the largest
single-GPU workload, and the one the bf16-MFMA-peak target is stated on.

Prints ONE JSON line.  `value` = samples/s through all segments' steps;
`roofline` = the matrix-product kernel (all three products of the step run
through it) priced against the dense bf16 MFMA peak, its duration measured live
with HIP events on the launch stream; `cpu_baseline` = the CPU oracle timed on a
bounded sample of the same workload.
"""

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2403_11204_amd import api, datagen  # noqa: E402

PEAK_TFLOPS = {api.BF16: 2516.6, api.F32: 157.3}     # dense MFMA peaks of MI355X
HBM_BYTES_PER_S = 8.0e12                             # published HBM3E rate of MI355X
# Bytes crossing the L2 boundary per matrix-product launch (read + written), average over the 16 launches of
# one step of the default workload: rocprofv3 FETCH_SIZE / WRITE_SIZE passes scaled by a 1 GiB copy kernel in
# the same process (profiles/comparison_config_gemm_hbm_traffic.md).  Valid for the kernel those passes ran;
# set to None whenever csrc/gemm.hip changes until the passes are repeated.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {4: 5.19e9}
MSE, CE = api.MSE_SIL, api.SOFTMAX_XENT
ALL, LAST = api.RELU_ALL, api.RELU_HIDDEN_IDENTITY_LAST

# name, dtype, batch, classes, samples, optimiser, segments: (widths, act, loss, label dist, label seed)
CONFIGS = {
    0: dict(name="tiny 784-128-64 | 64-64-47 fp32", dtype=api.F32, batch=64, classes=47, lr=0.01, mom=0.0, streams=False, graph=True,
            segs=[([784, 128, 64], ALL, MSE, api.UNIFORM_PM1, 7), ([64, 64, 47], LAST, CE, None, None)]),
    1: dict(name="paper-shaped 784-1024-1024-512 | 512-1024-1024-47 fp32", dtype=api.F32, batch=256, classes=47, lr=0.01,
            mom=0.9, streams=True, graph=True,
            segs=[([784, 1024, 1024, 512], ALL, MSE, api.NORMAL, 11), ([512, 1024, 1024, 47], LAST, CE, None, None)]),
    2: dict(name="wide 784-4096-4096-2048 | 2048-4096-4096-47 bf16", dtype=api.BF16, batch=1024, classes=47, lr=0.01,
            mom=0.9, streams=True, graph=True,
            segs=[([784, 4096, 4096, 2048], ALL, MSE, api.BINARY_PM1, 13), ([2048, 4096, 4096, 47], LAST, CE, None, None)]),
    3: dict(name="deep 12x8192 in 4 segments on 4 streams bf16", dtype=api.BF16, batch=4096, classes=100, lr=0.01, mom=0.9,
            streams=True,
            segs=[([784, 8192, 8192, 8192], ALL, MSE, api.NORMAL, 21), ([8192, 8192, 8192, 8192], ALL, MSE, api.NORMAL, 22),
                  ([8192, 8192, 8192, 8192], ALL, MSE, api.NORMAL, 23), ([8192, 8192, 8192, 100], LAST, CE, None, None)]),
    4: dict(name="comparison 784-16384-16384-16384 | 16384-16384-16384-1000 bf16", dtype=api.BF16, batch=8192, classes=1000,
            lr=0.01, mom=0.9, streams=False,
            segs=[([784, 16384, 16384, 16384], ALL, MSE, api.UNIFORM_PM1, 31),
                  ([16384, 16384, 16384, 1000], LAST, CE, None, None)]),
    # the network of the paper's own experiment (Sec. 3): 784-80-60 | 60-60-60-47, batch 1410, labels 10 * U(0,1)
    5: dict(name="paper Sec. 3 network 784-80-60 | 60-60-60-47 fp32", dtype=api.F32, batch=1410, classes=47, lr=0.01, mom=0.9,
            streams=True, graph=True, kappa=10.0,
            segs=[([784, 80, 60], ALL, MSE, api.UNIFORM01, 3), ([60, 60, 60, 47], LAST, CE, None, None)]),
}
E2E_WIDTHS = [784, 16384, 16384, 16384, 16384, 16384, 1000]


def gemm_flops_per_sample(widths):
    P = sum(widths[i] * widths[i + 1] for i in range(len(widths) - 1))
    return 6 * P - 2 * widths[0] * widths[1]


def build_segments(cfg, n_batches, only=None):
    """Handles, label tables and per-segment inputs for n_batches resident batches (only: that segment alone)."""
    dt, B, classes = cfg["dtype"], cfg["batch"], cfg["classes"]
    tdt = torch.bfloat16 if dt == api.BF16 else torch.float32
    ys, X0 = [], []
    for i in range(n_batches):
        X, y = datagen.class_mean_inputs(B, classes, dim=784, seed=1, first=i * B)
        X0.append(torch.from_numpy(X).cuda().to(tdt).contiguous())
        ys.append(torch.from_numpy(y).cuda())
    segs, inputs = [], []
    prev_table = None
    for si, (widths, act, loss, dist, seed) in enumerate(cfg["segs"]):
        table = None
        if loss == MSE and (only is None or si == only or si + 1 == only):
            table = api.make_synthetic_labels(seed, classes, widths[-1], dist, cfg.get("kappa", 1.0), api.F32)
        if only is not None and si != only:
            if si + 1 == only:          # the one table the wanted segment's inputs are made from
                prev_table = table
            continue
        seg = api.Segment(widths, act, loss, max_batch=B, dtype=dt, lr=cfg["lr"], momentum=cfg["mom"])
        seg.init(100 + si)
        if cfg.get("graph"):        # launch-bound sizes: replay the captured launch sequence of a step
            seg.set_graph(True)
        if cfg.get("fused"):        # optimiser step inside the weight-gradient products (pays on short products)
            seg.set_fused_update(cfg["fused"])
        if cfg.get("overlap"):      # segments stepped one after another: the update tail of one runs beside the next
            seg.set_overlap(True)
        if si == 0:
            inputs.append(X0)
        else:   # an interior/final segment sees the previous cut's label of the class plus noise (sigma 0.05)
            inputs.append([api.make_segment_inputs(5 + si, prev_table, ys[i], i * B, 0.05, dt) for i in range(n_batches)])
        if loss == MSE:
            prev_table = table
            seg.set_labels(table)
        segs.append(seg)
    if only is not None:
        prev_table = None
        if only != 0:
            del X0
    return segs, inputs, ys


def run_steps(segs, inputs, ys, streams, k0, k):
    for it in range(k0, k0 + k):
        bi = it % len(ys)
        if streams:
            for seg, xin, st in zip(segs, inputs, streams):
                with torch.cuda.stream(st):
                    seg.step(xin[bi], ys[bi], want_loss=True)
        else:
            for seg, xin in zip(segs, inputs):
                seg.step(xin[bi], ys[bi], want_loss=True)


def time_workload(segs, inputs, ys, use_streams, steps, warmup, profile=True):
    """Returns (wall ms/step, event ms/step, per-segment (gemm ms, launches, flops))."""
    streams = [torch.cuda.Stream() for _ in segs] if use_streams else None
    cur = torch.cuda.current_stream()
    if streams:
        for st in streams:
            st.wait_stream(cur)
    run_steps(segs, inputs, ys, streams, 0, warmup)
    torch.cuda.synchronize()
    if profile:
        for s in segs:
            s.profile_enable(steps * 3 * s.L + 8)     # event pairs created before the clock starts
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()
    run_steps(segs, inputs, ys, streams, warmup, steps)
    if streams:
        for st in streams:
            cur.wait_stream(st)
    for s in segs:
        s.join()              # updates that the last steps left running (overlap on) belong to the timed region
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    prof = [s.profile_read() for s in segs] if profile else None
    for s in segs:
        s.profile_enable(False)
    return wall_ms / steps, ev0.elapsed_time(ev1) / steps, prof


def cpu_baseline(cfg, rows):
    """The CPU oracle, as it stands, on a reduced batch of the same workload (all segments, full widths).

    A step of the oracle costs a part that does not depend on the batch (rounding every weight to bf16, the float64
    update of every parameter) plus a part per row (the matrix products).  Two steps are timed, on rows/4 and on rows
    rows, and the two parts separated from them, so that the reader can scale: `value` is what was measured at `rows`
    rows; `at_full_batch` extrapolates the same two costs to the configuration's batch."""
    from oracle import rng as orng
    from oracle import segment as osg
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    mode = "bf16" if cfg["dtype"] == api.BF16 else "fp32"
    classes = cfg["classes"]
    small = max(1, rows // 4)
    X, y = datagen.class_mean_inputs(rows, classes, dim=784, seed=1)
    t_small, t_rows, prev = 0.0, 0.0, None
    for si, (widths, act, loss, dist, seed) in enumerate(cfg["segs"]):
        o = osg.Segment(widths, act, loss, lr=cfg["lr"], momentum=cfg["mom"], mode=mode)
        for l, (W, b) in enumerate(datagen.uniform_weights(widths, 100 + si)):
            o.set_params(l, W, b)
        xin = X if si == 0 else orng.make_segment_inputs(5 + si, prev, y, 0, 0.05)
        table = None
        if loss == MSE:
            table = orng.make_synthetic_labels(seed, classes, widths[-1], dist, cfg.get("kappa", 1.0))
            prev = table
        t0 = time.perf_counter()
        o.step(xin[:small], y[:small], table)
        t1 = time.perf_counter()
        o.step(xin, y, table)
        t2 = time.perf_counter()
        t_small += t1 - t0
        t_rows += t2 - t1
        del o
    per_row = max(t_rows - t_small, 0.0) / max(rows - small, 1)
    fixed = max(t_rows - per_row * rows, 0.0)
    B = cfg["batch"]
    return {"value": rows / t_rows, "unit": "samples/s", "cores": int(cores), "kind": "oracle", "rows": rows,
            "seconds": t_rows, "fixed_seconds_per_step": fixed, "seconds_per_row": per_row,
            "product_share_of_step": per_row * rows / t_rows if t_rows > 0 else None,
            "at_full_batch": {"batch": B, "samples_per_s": B / (fixed + per_row * B), "kind": "extrapolated from the two costs"},
            "sample": "one step of every segment at full widths on %d rows (%.1f s of CPU time; a %d-row step before it, "
                      "%.1f s, separates the batch-independent cost from the per-row cost); the oracle's matrix products "
                      "are numpy float64 products, i.e. the host's BLAS on %d threads" % (rows, t_rows, small, t_small, int(cores))}


def measure_segment_peaks(cfg, steps=3):
    """Peak device memory of segment-wise training, measured: every segment is built, stepped a few times and freed
    on its own, which is how the method trains (only one partition's parameters, optimiser state and activations
    are resident at a time)."""
    peaks = []
    for si in range(len(cfg["segs"])):
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        torch.cuda.reset_peak_memory_stats()
        base = torch.cuda.memory_allocated()
        sub = dict(cfg)
        segs, inputs, ys = build_segments(sub, n_batches=1, only=si)
        for _ in range(steps):
            segs[0].step(inputs[0][0], ys[0], want_loss=True)
        segs[0].join()
        torch.cuda.synchronize()
        peaks.append(int(torch.cuda.max_memory_allocated() - base))
        del segs, inputs, ys
    torch.cuda.empty_cache()
    return peaks


def pipeline_phases(cfg, reps=5):
    """The other phases of the paper's procedure at the main workload's shape (Sec. 2, Sec. 5), timed with events on
    the current stream: the forward-only pass that stores the left partition's response, and one recovery step (left
    forward, input gradient of the frozen right partition, left step from that gradient)."""
    dt, B, classes = cfg["dtype"], cfg["batch"], cfg["classes"]
    (wl, al, ll, dist, seed), (wr, ar, lr_, _, _) = cfg["segs"][0], cfg["segs"][-1]
    left = api.Segment(wl, al, ll, max_batch=B, dtype=dt, lr=cfg["lr"], momentum=cfg["mom"])
    right = api.Segment(wr, ar, lr_, max_batch=B, dtype=dt, lr=cfg["lr"], momentum=cfg["mom"], input_grad=True)
    left.init(100)
    right.init(101)
    left.set_labels(api.make_synthetic_labels(seed, classes, wl[-1], dist, cfg.get("kappa", 1.0), api.F32))
    X, y = datagen.class_mean_inputs(B, classes, dim=wl[0], seed=1)
    tdt = torch.bfloat16 if dt == api.BF16 else torch.float32
    Xd, yd = torch.from_numpy(X).cuda().to(tdt).contiguous(), torch.from_numpy(y).cuda()
    resp = torch.empty((B, wl[-1]), dtype=tdt, device="cuda")

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def recovery():
        left.forward(Xd, out=resp)
        d_resp, _ = right.input_grad(resp, yd)
        left.step_external(Xd, d_resp)

    fwd_ms = timed(lambda: left.forward(Xd, out=resp))
    rec_ms = timed(recovery)
    P = lambda w: sum(w[i] * w[i + 1] for i in range(len(w) - 1))
    fwd_fl = 2.0 * P(wl) * B
    # recovery: left forward twice (response, then inside the step), right forward + every data gradient, left backward
    rec_fl = (2.0 * P(wl) + 2.0 * P(wl) + 4.0 * P(wr) + (4.0 * P(wl) - 2.0 * wl[0] * wl[1])) * B
    out = {"store_response": {"segment": wl, "ms_per_batch": fwd_ms, "samples_per_s": B / (fwd_ms * 1e-3),
                              "tflops": fwd_fl / (fwd_ms * 1e-3) / 1e12},
           "recovery_step": {"left": wl, "right_frozen": wr, "ms_per_step": rec_ms, "samples_per_s": B / (rec_ms * 1e-3),
                             "tflops": rec_fl / (rec_ms * 1e-3) / 1e12}}
    del left, right
    torch.cuda.empty_cache()
    return out


def quick_config(cid, steps, warmup):
    """ms per step, TFLOP/s and fractions of another configuration, measured the same way as the main workload."""
    cfg = dict(CONFIGS[cid])
    cfg["overlap"] = False
    if cfg.get("graph"):
        cfg["fused"] = 2
    segs, inputs, ys = build_segments(cfg, n_batches=2)
    torch.cuda.synchronize()
    if cfg.get("graph"):
        with torch.cuda.stream(torch.cuda.Stream()):
            wall_ms, ev_ms, _ = time_workload(segs, inputs, ys, cfg["streams"], steps, warmup, profile=False)
            _, _, prof = time_workload(segs, inputs, ys, False, max(steps // 4, 10), 2)
    else:
        wall_ms, ev_ms, prof = time_workload(segs, inputs, ys, cfg["streams"], steps, warmup)
    ms = max(wall_ms, ev_ms) if not cfg["streams"] else wall_ms
    B, peak = cfg["batch"], PEAK_TFLOPS[cfg["dtype"]]
    flops_step = sum(gemm_flops_per_sample(s[0]) for s in cfg["segs"]) * B
    gemm_ms, gemm_fl = sum(p[0] for p in prof), sum(p[2] for p in prof)
    n_params = sum(sum((w[i] + 1) * w[i + 1] for i in range(len(w) - 1)) for w in (s[0] for s in cfg["segs"]))
    out = {"workload": cfg["name"], "global_batch": B, "steps": steps, "ms_per_step": ms, "samples_per_s": B / (ms * 1e-3),
           "step_tflops": flops_step / (ms * 1e-3) / 1e12, "step_frac_of_mfma_peak": flops_step / (ms * 1e-3) / 1e12 / peak,
           # launch-by-launch events overlap when the segments run concurrently: no per-kernel rate then
           "gemm_tflops": gemm_fl / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 and (cfg.get("graph") or not cfg["streams"]) else None,
           "launch": "hip graph replay" if cfg.get("graph") else "eager", "fused_update": cfg.get("fused", 0),
           "concurrent_streams": len(segs) if cfg["streams"] else 1,
           # the other roof: every parameter streams through the step once per product that reads it and through the
           # update (24 B with momentum in bf16 mode: g, v, w read; v, w, bf16 copy, transposed copy written)
           "param_bytes_per_step_algorithmic": 24 * n_params if cfg["dtype"] == api.BF16 else 28 * n_params,
           "hbm_floor_ms": (24 if cfg["dtype"] == api.BF16 else 28) * n_params / HBM_BYTES_PER_S * 1e3}
    if cfg["streams"]:
        # the same segments one after another on one stream, update tails overlapped (what `--config N --serial` times)
        if not cfg.get("graph"):
            for seg in segs:
                seg.set_overlap(True)
        w2, e2, _ = time_workload(segs, inputs, ys, False, steps, warmup, profile=False)
        ms2 = max(w2, e2)
        out["one_stream"] = {"ms_per_step": ms2, "samples_per_s": B / (ms2 * 1e-3), "step_tflops": flops_step / (ms2 * 1e-3) / 1e12,
                             "step_frac_of_mfma_peak": flops_step / (ms2 * 1e-3) / 1e12 / peak}
    del segs, inputs, ys
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", type=int, default=4, choices=sorted(CONFIGS))
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--no-e2e", action="store_true", help="skip the end-to-end backprop comparison (config 4)")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other configurations (config 4)")
    ap.add_argument("--cpu-rows", type=int, default=None)
    ap.add_argument("--calib-copy", action="store_true",
                    help="first run one plain 1 GiB -> 1 GiB elementwise copy kernel (scale reference for HBM byte counters)")
    ap.add_argument("--graph", action="store_true", help="replay captured steps on a configuration that launches eagerly by default")
    ap.add_argument("--eager", action="store_true", help="configs 0-2: launch every kernel of a step instead of replaying graphs")
    ap.add_argument("--fused", type=int, nargs="?", const=1, default=0, help="apply the update in the epilogue of the weight-gradient products")
    ap.add_argument("--unfused", action="store_true", help="configs 0-2 and 5: separate update launches instead of the fused update")
    ap.add_argument("--events-apart", action="store_true",
                    help="time the steps without per-launch events and the matrix products in a second pass (as the graph configs do)")
    ap.add_argument("--serial", action="store_true", help="run the segments one after another on one stream (configs 1, 2, 3, 5 default to a stream each)")
    ap.add_argument("--no-overlap", action="store_true",
                    help="end every step by waiting for its parameter updates (slp_segment_set_overlap off)")
    ap.add_argument("--concurrent", action="store_true", help="run the segments at the same time on a stream each (the default of configs 1, 2, 3, 5)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (segments are independent jobs; no collectives exist): use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    cfg = dict(CONFIGS[args.config])
    if cfg.get("graph"):         # small and mid-size layers: the update inside the weight-gradient products (rule 2)
        cfg["fused"] = 2
    if args.graph:
        cfg["graph"] = True
    if args.fused:
        cfg["fused"] = args.fused
    if args.unfused:
        cfg["fused"] = False
    if args.serial:
        cfg["streams"] = False
    if args.concurrent:
        cfg["streams"] = True
    cfg["overlap"] = (len(cfg["segs"]) > 1 and not cfg["streams"] and (not cfg.get("graph") or args.eager)
                      and not args.no_overlap)
    big = args.config in (3, 4)
    steps = args.steps if args.steps is not None else (20 if big else 200)
    warmup = args.warmup if args.warmup is not None else (3 if big else 20)
    dt, B = cfg["dtype"], cfg["batch"]

    if args.calib_copy:
        src = torch.rand(1 << 28, dtype=torch.float32, device="cuda")       # 1 GiB
        dst = torch.empty_like(src)
        torch.mul(src, 1.0, out=dst)                                         # one kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    segs, inputs, ys = build_segments(cfg, n_batches=2 if big else 8)
    torch.cuda.synchronize()
    if cfg.get("graph") and not args.eager:
        # graphs cannot be captured on the null stream; the matrix products are timed in a second, eager pass
        # (launch-by-launch events and replayed graphs exclude each other)
        with torch.cuda.stream(torch.cuda.Stream()):
            wall_ms, ev_ms, _ = time_workload(segs, inputs, ys, cfg["streams"], steps, warmup, profile=False)
            prof_steps = max(steps // 4, 10)
            _, _, prof = time_workload(segs, inputs, ys, False, prof_steps, 2)
    elif args.events_apart:
        wall_ms, ev_ms, _ = time_workload(segs, inputs, ys, cfg["streams"], steps, warmup, profile=False)
        prof_steps = max(steps // 2, 5)
        _, _, prof = time_workload(segs, inputs, ys, cfg["streams"], prof_steps, 2)
    else:
        prof_steps = steps
        wall_ms, ev_ms, prof = time_workload(segs, inputs, ys, cfg["streams"], steps, warmup)
    ms = max(wall_ms, ev_ms) if not cfg["streams"] else wall_ms
    flops_step = sum(gemm_flops_per_sample(s[0]) for s in cfg["segs"]) * B
    peak = PEAK_TFLOPS[dt]
    gemm_ms = sum(p[0] for p in prof)
    gemm_n = sum(p[1] for p in prof)
    gemm_fl = sum(p[2] for p in prof)
    achieved = gemm_fl / (gemm_ms * 1e-3) / 1e12 if gemm_ms > 0 else 0.0
    seg_bytes = [(s.param_bytes, s.workspace_bytes) for s in segs]
    out = {
        "metric": "segment_train_samples_per_s", "value": B / (ms * 1e-3), "unit": "samples/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if dt == api.BF16 else "f32", "data": "synthetic",
        "config": {"workload": cfg["name"], "global_batch": B, "classes": cfg["classes"],
                   "segments": [s[0] for s in cfg["segs"]], "optimizer": "sgd lr %g momentum %g" % (cfg["lr"], cfg["mom"]),
                   "concurrent_streams": len(segs) if cfg["streams"] else 1,
                   "launch": "hip graph replay" if cfg.get("graph") and not args.eager else "eager",
                   "update_overlap": bool(cfg["overlap"]), "fused_update": cfg.get("fused", 0)},
        "step_tflops": flops_step / (ms * 1e-3) / 1e12,
        "step_frac_of_mfma_peak": flops_step / (ms * 1e-3) / 1e12 / peak,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                     "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(args.config), "kernel": "gemm_nt_big_kernel" if args.config in (3, 4) else "gemm_nt_kernel", "launches": gemm_n,
                     "avg_launch_ms": gemm_ms / max(gemm_n, 1), "flops_per_launch": gemm_fl / max(gemm_n, 1)},
        "segment_bytes": [{"params": p, "workspace": w} for p, w in seg_bytes],
        "peak_hbm_bytes_torch": int(torch.cuda.max_memory_allocated()),
    }
    if not cfg["streams"]:
        out["per_segment_gemm_ms"] = [p[0] / prof_steps for p in prof]
    # what the matrix pipe sustains on this chip with no memory traffic at all (register-only MFMA loop, ~50 ms)
    sustained, _ = api.probe_mfma_rate(dt, iters=20000 if dt == api.BF16 else 4000)
    out["roofline"]["sustained_mfma_only"] = sustained
    out["roofline"]["frac_of_sustained"] = achieved / sustained

    segs = inputs = None          # everything below runs with the main workload's segments freed
    torch.cuda.empty_cache()
    if args.config == 4 and not args.no_e2e:
        # conventional end-to-end backprop through all six layers on the same GPU, same library
        torch.cuda.reset_peak_memory_stats()
        e2e = api.Segment(E2E_WIDTHS, LAST, CE, max_batch=B, dtype=dt, lr=cfg["lr"], momentum=cfg["mom"])
        e2e.init(200)
        X0 = []
        for i in range(2):
            X, _ = datagen.class_mean_inputs(B, cfg["classes"], dim=784, seed=1, first=i * B)
            X0.append(torch.from_numpy(X).cuda().to(torch.bfloat16).contiguous())
        ks = max(3, steps // 2)
        w_ms, e_ms, p = time_workload([e2e], [X0], ys, False, ks, 2)
        m = max(w_ms, e_ms)
        fl = gemm_flops_per_sample(E2E_WIDTHS) * B
        out["end_to_end_baseline"] = {
            "widths": E2E_WIDTHS, "ms_per_step": m, "samples_per_s": B / (m * 1e-3), "tflops": fl / (m * 1e-3) / 1e12,
            "params_bytes": e2e.param_bytes, "workspace_bytes": e2e.workspace_bytes,
            "peak_hbm_bytes_torch": int(torch.cuda.max_memory_allocated()),
            "segmentwise_ms_per_step": ms}
        del e2e, X0
        torch.cuda.empty_cache()
        # the method's memory claim (Sec. 2.1), measured: each segment built, trained and freed on its own
        peaks = measure_segment_peaks(cfg)
        out["end_to_end_baseline"]["segmentwise_peak_bytes_measured"] = max(peaks)
        out["end_to_end_baseline"]["segmentwise_peak_bytes_per_segment"] = peaks
        out["end_to_end_baseline"]["segmentwise_peak_bytes_arithmetic"] = max(p_ + w_ for p_, w_ in seg_bytes)
        out["end_to_end_baseline"]["both_segments_resident_peak_bytes"] = out["peak_hbm_bytes_torch"]

    if args.config == 4 and not args.no_others:
        # the other configurations, short runs (their own lines: --config N): wide, deep, paper-shaped, the paper's own network
        ys = None
        torch.cuda.empty_cache()
        out["other_configs"] = [quick_config(2, 200, 20), quick_config(3, 10, 3), quick_config(1, 500, 50), quick_config(5, 500, 50)]
        # the forward-only pass and the recovery step of the paper's procedure at this configuration's shape
        out["pipeline_phases"] = pipeline_phases(cfg)

    if not args.no_cpu:
        rows = args.cpu_rows or {0: 64, 1: 256, 2: 256, 3: 256, 4: 256, 5: 1410}[args.config]
        out["cpu_baseline"] = cpu_baseline(cfg, rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
