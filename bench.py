#!/usr/bin/env python3
"""Benchmark of the mixed-precision stacked-LSTM training step on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic
input: for every simulated worker fprop + loss + BPTT, then grad_average, the
learning-rate schedule and master_update.  Inputs are resident in HBM before
the timed region starts.  Prints ONE JSON line on stdout.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"fp16": 2500.0, "bf16": 2500.0, "fp32": 157.3}   # dense MFMA (fp32: vector ALU)
PEAK_HBM_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def gemm_flops_per_step(w) -> float:
    """Algorithmic GEMM work of one step: 6 * weights * B * T per worker
    (forward, data gradient, weight gradient), minus the input-data gradient of
    layer 0 when its input is data rather than an embedding."""
    G = 4 * w.hidden
    tot = 0.0
    for l, i_l in enumerate(w.layer_input_dims):
        tot += 6.0 * G * (i_l + w.hidden)
        if l == 0 and w.vocab == 0:
            tot -= 2.0 * G * i_l
    return tot * w.batch * w.seq_len * w.n_workers


def measured_traffic(workload: str, kernel_class: str):
    """HBM bytes per launch of one kernel class as measured with rocprofv3's
    FETCH_SIZE and WRITE_SIZE counters (scaled by the copy-kernel calibration);
    read from the committed counter summary of this workload, (None, None) if
    there is no summary for it.  Counters cannot be collected from inside this
    process: the second value says which file and which build the figure is
    from, so that it can be told apart from what this run measured itself."""
    rel = os.path.join("profiles", f"{workload}_hbm_traffic.txt")
    value, build = None, "unknown build"
    try:
        with open(os.path.join(ROOT, rel)) as f:
            for line in f:
                p = line.split()
                if len(p) == 3 and p[0] == "class" and p[1] == kernel_class:
                    value = float(p[2])
                if len(p) >= 3 and p[0] == "#" and p[1] == "build:":
                    build = p[2]
    except OSError:
        return None, None
    return value, (f"{rel} (rocprofv3 counters of build {build}; not measured in this run)" if value is not None else None)


def measured_peaks(hip, torch, dtype: str):
    """What this GPU sustains on the two plain patterns the rooflines are named after, measured here:
    a register-resident MFMA loop (on constant operands and on N(0,1) operands: power management
    makes the rate depend on the operand values) and a plain 1 GiB device copy."""
    dev = torch.device("cuda:0")
    res = {}
    if dtype in ("fp16", "bf16"):
        tdt, code = (torch.float16, hip.DTYPE_FP16) if dtype == "fp16" else (torch.bfloat16, hip.DTYPE_BF16)
        n = 256 * 512 * 2 * 8
        sink = torch.zeros(1, dtype=torch.float32, device=dev)
        gen = torch.Generator(device="cpu").manual_seed(0)
        for label, ops in (("constant", torch.full((n,), 0.5, dtype=tdt, device=dev)),
                           ("normal", torch.randn(n, generator=gen).to(tdt).to(dev))):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            hip.lstm_debug_mfma_rate(code, ops, 2000, sink)            # warm-up
            e0.record()
            flops = hip.lstm_debug_mfma_rate(code, ops, 40000, sink)
            e1.record()
            torch.cuda.synchronize()
            res[f"mfma_{label}_operands_tflops"] = flops / (e0.elapsed_time(e1) * 1e-3) / 1e12
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    res["device_copy_gbs"] = 5 * 2.0 * src.numel() * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    return res


def cpu_baseline(w, budget_flops=6.0e12):
    """Time the CPU oracle (as it stands) on a bounded sample of the workload:
    same model and batch, sequence shortened so the fp64 work stays near
    budget_flops; the cost is linear in the number of time steps."""
    import numpy as np
    from oracle import lstm_oracle as orc
    from tests import parity_util as pu
    per_t = gemm_flops_per_step(w) / w.seq_len / w.n_workers
    T_s = int(max(1, min(w.seq_len, budget_flops // max(per_t, 1.0))))
    ws = w.with_(seq_len=T_s, n_workers=1)
    master0, xs, ys = pu.inputs_for(ws)
    shapes = pu.oracle_shapes(ws)
    t0 = time.perf_counter()
    out = orc.training_step(master0.astype(np.float64), shapes, ws.num_layers,
                            [(xs[0] if ws.vocab else xs[0].astype(np.float64), ys[0])], ws.head, ws.loss_scale,
                            ws.lr0, ws.momentum)
    dt = time.perf_counter() - t0
    one_thread = None
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        if dt < 4.0:                            # the small workloads: the same sample on one thread as well
            with threadpool_limits(limits=1):
                t0 = time.perf_counter()
                orc.training_step(master0.astype(np.float64), shapes, ws.num_layers,
                                  [(xs[0] if ws.vocab else xs[0].astype(np.float64), ys[0])], ws.head, ws.loss_scale,
                                  ws.lr0, ws.momentum)
                one_thread = ws.batch * T_s / (time.perf_counter() - t0)
    except ImportError:
        cores = os.cpu_count() or 1
    return {"value": ws.batch * T_s / dt, "unit": "sample-timesteps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{w.name} model and batch, first {T_s} of {w.seq_len} time steps, 1 worker, one fwd+BPTT+update "
                      f"in fp64 numpy ({dt:.2f} s)", "one_thread_value": one_thread, "loss": out["losses"][0]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--dtype", default=None, choices=["fp16", "bf16", "fp32"],
                    help="storage type override (bf16: no loss scaling needed, static scale 1; fp32: the paper's "
                         "all-single-precision baseline mode, no loss scaling)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=0,
                    help="streams the simulated workers are spread over (0: 4 when there are several workers, else 1)")
    ap.add_argument("--one-by-one", action="store_true",
                    help="run the simulated workers' fprop/BPTT one after another instead of stacked into one call")
    ap.add_argument("--eager", action="store_true",
                    help="enqueue every launch from the host in the timed region instead of replaying a HIP graph")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run 5 plain device copies of 1 GiB and exit (reference for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU only (no collectives are part of it); "
            f"--gpus {args.gpus} is not supported. value is one MI355X's throughput.")
        sys.exit(2)

    import numpy as np
    import torch
    import workloads as wl
    import paper_1912_00286_amd as hip
    from tests import parity_util as pu

    hip.load_library()                      # no fallback: fails loudly if the HIP library is absent
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        n = 1 << 29                         # 2^29 fp16 elements = 1 GiB read + 1 GiB written per copy
        src = torch.ones(n, dtype=torch.float16, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "5 device copies", "bytes_read_each": 2 * n, "bytes_written_each": 2 * n}))
        return
    w = wl.CONFIGS[args.workload] if args.workload in wl.CONFIGS else wl.EXTRA[args.workload]
    if args.dtype and args.dtype != w.dtype:
        w = w.with_(dtype=args.dtype, **({"loss_scale": 1.0, "dynamic_scale": False} if args.dtype in ("bf16", "fp32") else {}))
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    log(f"[bench] workload {w.name}: L={w.num_layers} H={w.hidden} T={w.seq_len} B={w.batch} N={w.n_workers} {w.dtype}")

    master0, xs, ys = pu.inputs_for(w)
    n_streams = args.streams if args.streams > 0 else (4 if w.n_workers > 1 else 1)
    ts = None
    if w.n_workers > 1 and not args.one_by_one:
        try:                                    # all workers' micro-batches stacked into one call per direction
            ts = pu.make_step(w, master0, dev, batched=True)
        except hip.LstmError as e:
            log(f"[bench] stacked form not available for this shape ({e}); running the workers one by one")
    if ts is None:
        ts = pu.make_step(w, master0, dev, n_streams=n_streams)
    dx, dy = pu.device_batches(w, xs, ys, ts.lp_dtype, dev)
    if ts.batched:
        dx, dy = ts.stack_workers(dx, dy)
    del xs, ys

    # fprop + BPTT of every worker and the gradient average are recorded once as a HIP graph (this
    # runs nothing); a step is then one graph launch plus master_update with that step's rate
    if not args.eager:
        ts.capture(dx, dy)
    run_step = (lambda lr: ts.step(dx, dy, lr)) if args.eager else ts.step_captured
    k = 0
    for _ in range(args.warmup):
        run_step(pu.lr_for(w, k)); k += 1
    torch.cuda.synchronize()
    good0, scale0 = int(ts.good_steps.item()), float(ts.loss_scale.item())
    log(f"[bench] warm-up done, loss {ts.losses[0].item():.5f}, loss scale {scale0}")

    # ---- timed region: exactly K steps, nothing but enqueues inside
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step(pu.lr_for(w, k)); k += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    overflow_steps = None
    if w.dynamic_scale:
        overflow_steps = args.steps - (int(ts.good_steps.item()) - good0)
    elif int(ts.found_inf.item()):
        overflow_steps = "last step overflowed"
    loss_after = float(ts.losses[0].item())
    assert np.isfinite(loss_after), "loss is not finite"
    ms_per_step = dt / args.steps * 1e3
    sample_steps = w.n_workers * w.batch * w.seq_len
    value = sample_steps * args.steps / dt

    # ---- same K steps again with HIP events around every launch (per-class durations)
    hip.lstm_timing_enable(True)
    for _ in range(args.steps):
        ts.step(dx, dy, pu.lr_for(w, k)); k += 1
    torch.cuda.synchronize()
    classes = {name: hip.lstm_timing_read(i) for i, name in enumerate(hip.KERNEL_CLASSES)}
    hip.lstm_timing_enable(False)
    for c in classes.values():
        c["avg_us"] = 1e3 * c["total_ms"] / max(c["launches"], 1)
        c["ms_per_step"] = c["total_ms"] / args.steps
    dom = max(classes, key=lambda n: classes[n]["total_ms"])
    c = classes[dom]
    secs = c["total_ms"] * 1e-3
    peak_fl = PEAK_TFLOPS[w.dtype]
    # A GEMM launch whose arithmetic intensity (flops per algorithmic byte: every operand read once,
    # the result written once) lies below the chip's ridge point peak_flops / peak_bytes is bound by
    # the memory roofline, not by the matrix cores: the per-time-step recurrent GEMMs at batch 256 are.
    intensity = (c["flops"] / c["bytes"]) if c["bytes"] else float("inf")
    ridge = peak_fl * 1e12 / (PEAK_HBM_GBS * 1e9)
    if dom.startswith("gemm") and intensity >= ridge:
        achieved = c["flops"] / secs / 1e12
        roof = {"bound": "mfma" if w.dtype != "fp32" else "alu", "achieved": achieved, "peak": peak_fl,
                "unit": "TFLOP/s", "frac": achieved / peak_fl, "traffic": None}
    else:
        achieved = c["bytes"] / secs / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None}
    if dom.startswith("gemm"):
        roof.update({"flops_per_byte": intensity, "ridge_flops_per_byte": ridge,
                     "tflops": c["flops"] / secs / 1e12, "mfma_frac": c["flops"] / secs / 1e12 / peak_fl})
    roof["traffic"], roof["traffic_source"] = measured_traffic(w.name, dom)
    roof.update({"kernel_class": dom, "algorithmic_bytes_per_launch": c["bytes"] / max(c["launches"], 1), "launches_per_step": c["launches"] / args.steps, "avg_launch_us": c["avg_us"]})
    gemm_ms = classes["gemm_batched"]["total_ms"] + classes["gemm_step"]["total_ms"]
    gemm_fl = classes["gemm_batched"]["flops"] + classes["gemm_step"]["flops"]

    out = {
        "metric": "training timesteps/sec (fwd+BPTT+update) per MI355X; % peak fp16 MFMA",
        "value": value, "unit": "sample-timesteps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {"fp16": "f16", "bf16": "bf16", "fp32": "f32"}[w.dtype], "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.num_layers}-layer LSTM, input {w.embed_dim if w.vocab else w.input_dim}, "
                               f"hidden {w.hidden}, seq {w.seq_len}, batch {w.batch}, {w.n_workers} worker(s), "
                               f"{hip.lstm_param_count(pu.make_cfg(w))} params, {w.dtype} storage / fp32 accumulate+master, "
                               f"{'dynamic' if w.dynamic_scale else 'static'} loss scale"},
        "samples_per_s": w.n_workers * w.batch * args.steps / dt,
        "sequential_steps_per_s": w.seq_len * w.num_layers * w.n_workers * args.steps / dt,
        "step_mfma_frac": gemm_flops_per_step(w) / (ms_per_step * 1e-3) / 1e12 / PEAK_TFLOPS[w.dtype],
        "gate_gemm_mfma_frac": (gemm_fl / (gemm_ms * 1e-3) / 1e12 / PEAK_TFLOPS[w.dtype]) if gemm_ms > 0 else None,
        "worker_streams": ts.n_streams, "workers_stacked": ts.batched,
        "launch": "eager" if args.eager else "hip_graph (fprop+BPTT+grad_average) + master_update",
        "overflow_steps": overflow_steps, "loss_scale": float(ts.loss_scale.item()), "loss": loss_after,
        "roofline": roof,
        "kernel_classes": {n: {"ms_per_step": round(v["ms_per_step"], 4), "launches_per_step": v["launches"] / args.steps,
                               "avg_us": round(v["avg_us"], 2),
                               "tflops": (v["flops"] / (v["total_ms"] * 1e-3) / 1e12) if v["flops"] and v["total_ms"] else None,
                               "gbs": (v["bytes"] / (v["total_ms"] * 1e-3) / 1e9) if v["bytes"] and v["total_ms"] else None}
                           for n, v in classes.items()},
    }
    del ts, dx, dy
    torch.cuda.empty_cache()
    out["measured_peaks"] = measured_peaks(hip, torch, w.dtype)
    if not args.no_cpu_baseline:
        log("[bench] timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
