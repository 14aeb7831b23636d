#!/usr/bin/env python3
"""Benchmark of the TWA projected-gradient step on one MI355X.

One "step" is one pass of the whole hot path over one synthetic gradient:
    s = P^T g   (twa_project)      then      g~ = P s, w -= lr g~   (twa_expand_update)
enqueued back to back on one stream, s staying on the device.  The workload is the
ResNet-50-sized configuration the metric is quoted on: D = 25,557,032, n = 100, P stored as int8
codes with one fp32 absmax scale per 128 elements.  P is produced by the library itself from a
synthetic checkpoint trajectory (twa_build_basis, then twa_quantize); all inputs are resident in
HBM before the timed region starts.

Prints ONE JSON line.  `value` = projected steps/s; `p_stream_GBps` = steps/s x 2 x (bytes of P);
`roofline` = the slower of the two kernels against the 8 TB/s HBM peak, its duration measured here
with device events on the stream the kernels run on; `cpu_baseline` = the fp64 oracle timed on the
host cores on a bounded sample of the same stored P.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
METRIC = "projected steps/s and P-stream HBM GB/s (% of peak), D=25.6M n=100 int8"
METRIC_LAYERWISE = "layer-wise coefficient-form steps/s (Alg. 1) and P-stream HBM GB/s (% of peak)"


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (profiles/hbm_traffic_*.txt), or None."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_imagenet_resnet50_int8.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        parts = line.split("#")[0].split()
        if len(parts) >= 3 and parts[0] == "traffic_bytes_per_launch" and parts[1] == kernel:
            return float(parts[2])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=1000,
                    help="untimed steps; the device needs ~0.5 s of this load before the step time settles")
    ap.add_argument("--workload", default="imagenet_resnet50", help="name in synth.WORKLOADS")
    ap.add_argument("--storage", default="i8", choices=["f32", "bf16", "i8", "i4", "mm16", "mm8", "mm4", "mm3", "mm2", "mm1"],
                    help="mm16 .. mm1: the paper's per-layer min-max codes of that many bits (layer-wise mode only)")
    ap.add_argument("--mode", default="whole", choices=["whole", "layerwise"],
                    help="whole: the headline step (orthonormal basis, s = P^T g, w -= lr P s).  layerwise: Alg. 1 as "
                         "written -- per-layer centre+normalise basis, coefficient step with weight decay, w = wbar + P beta")
    ap.add_argument("--D", type=int, default=0, help="override the parameter count (smoke runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known 1 GiB read + 1 GiB write) so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU library (no collectives, no sharding); run with --gpus 1. "
                 "How the path would shard over GPUs is described in the repository's design notes.")

    import numpy as np
    import torch
    from paper_2205_13104_amd import binding as twa
    from paper_2205_13104_amd import synth

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    twa.lib()   # fail loudly if the library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    wl = synth.WORKLOADS[args.workload]
    D = args.D or wl.D
    n = wl.n
    dtype = {"f32": twa.F32, "bf16": twa.BF16, "i8": twa.I8, "i4": twa.I4, "mm8": twa.U8MM, "mm4": twa.U4MM,
             "mm16": twa.U16MM, "mm3": twa.U3MM, "mm2": twa.U2MM, "mm1": twa.U1MM}[args.storage]
    layerwise = args.mode == "layerwise"
    if dtype in twa.MINMAX_TYPES and not layerwise:
        sys.exit("bench.py: the min-max formats exist for the layer-wise calls only (use --mode layerwise)")

    # ---- inputs: checkpoints -> orthonormal basis (in place) -> stored P ------------------------
    t0 = time.time()
    W = synth.checkpoints(wl, seed=args.seed, device=dev, D=D)
    w = W[:, :D].mean(dim=0).contiguous()                  # the plain average: starting point of TWA
    torch.cuda.synchronize()
    t1 = time.time()
    plan = None
    if layerwise:
        sizes = synth.workload_layers(wl.name) if D == wl.D else synth.layer_offsets(synth.random_layer_sizes(D, 12, 11))
        plan = twa.LayerPlan(sizes, D)
        P32, w, _ = twa.centre_normalise(W, D, plan, out=W, want_norms=False)     # w = wbar: Alg. 1 starts at the mean
        wbar = w.clone()
    else:
        if wl.name == "large":
            # this configuration's basis is built from 16 M-row panels (the calls a caller uses whose checkpoints
            # do not sit in memory at once; here they do, so the panels are views)
            P32, _ = twa.build_basis_panels(W, D, 1 << 24, out=W)
        else:
            P32, _ = twa.build_basis(W, D, out=W, want_R=False)
    torch.cuda.synchronize()
    t2 = time.time()
    if dtype == twa.F32:
        pm = twa.wrap_f32(P32, D)
    elif dtype in twa.MINMAX_TYPES:
        pm = twa.quantize_minmax(P32, D, plan, bits=twa.BITS_OF[dtype])
    else:
        pm = twa.quantize(P32, D, dtype)
    torch.cuda.synchronize()
    t3 = time.time()
    if dtype != twa.F32:
        del W, P32
        torch.cuda.empty_cache()
    log(f"[bench] {wl.name}: D={D} n={n} storage={args.storage}; generate {t1 - t0:.2f}s, "
        f"build_basis {t2 - t1:.3f}s, quantize {t3 - t2:.3f}s")
    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                                   # the calibration kernel: reads 2^30 B, writes 2^30 B
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    ring = [synth.gradient(D, wl.sigma_g, seed=args.seed, step=i, device=dev) for i in range(4)]
    lr = wl.lr
    lam = 1e-4                                  # weight decay of the coefficient form (layer-wise mode)
    if layerwise:
        L = plan.L
        beta = torch.zeros((L, n), dtype=torch.float32, device=dev)
        ws = twa.Workspace(twa.project_layers_workspace_bytes(n, L), device=dev)

        def step(i):
            twa.beta_step(pm, ring[i & 3], plan, beta, lr, lam, None, ws)
            twa.weights_from_beta(pm, beta, plan, wbar, w)
    else:
        s = torch.empty(n, dtype=torch.float32, device=dev)
        ws = twa.Workspace(twa.project_workspace_bytes(n), device=dev)

        def step(i):
            twa.project(pm, ring[i & 3], s, ws)
            twa.expand_update(pm, s, w, lr)

    # ---- the timed region: exactly K steps --------------------------------------------------------
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    wall0 = time.perf_counter()
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - wall0
    ms_total = e0.elapsed_time(e1)
    ms_per_step = max(ms_total, wall * 1e3) / args.steps    # never report less than the host saw
    steps_per_s = 1e3 / ms_per_step
    p_bytes = pm.stream_bytes
    p_stream_gbps = steps_per_s * 2 * p_bytes / 1e9

    # ---- per-kernel launch durations (device events around every launch, same stream) ----------
    K2 = min(args.steps, 200)

    def timed_each(fn):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K2)]
        for i, (a, b) in enumerate(evs):
            a.record()
            fn(i)
            b.record()
        torch.cuda.synchronize()
        return sum(a.elapsed_time(b) for a, b in evs) / K2

    if layerwise:
        ms_project = timed_each(lambda i: twa.beta_step(pm, ring[i & 3], plan, beta, lr, lam, None, ws))
        ms_expand = timed_each(lambda i: twa.weights_from_beta(pm, beta, plan, wbar, w))
        alg = {
            "twa_beta_step": p_bytes + 4 * D + 8 * n * L,           # P once + g + beta read and written
            "twa_weights_from_beta": p_bytes + 8 * D + 4 * n * L,   # P once + wbar read + w written + beta
        }
        dur = {"twa_beta_step": ms_project, "twa_weights_from_beta": ms_expand}
    else:
        ms_project = timed_each(lambda i: twa.project(pm, ring[i & 3], s, ws))
        ms_expand = timed_each(lambda i: twa.expand_update(pm, s, w, lr))
        alg = {
            "twa_project": p_bytes + 4 * D + 4 * n,                 # P once + g + s
            "twa_expand_update": p_bytes + 8 * D + 4 * n,           # P once + w read + w write + s
        }
        dur = {"twa_project": ms_project, "twa_expand_update": ms_expand}
    dom = max(dur, key=dur.get)
    achieved = alg[dom] / (dur[dom] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": read_traffic(dom),
                "algorithmic_bytes_per_launch": alg[dom], "avg_launch_ms": round(dur[dom], 5),
                "other_kernel": {"kernel": min(dur, key=dur.get), "avg_launch_ms": round(min(dur.values()), 5),
                                 "achieved": round(alg[min(dur, key=dur.get)] / (min(dur.values()) * 1e-3) / 1e9, 1)}}

    # ---- the read ceiling of this device, measured: plain non-temporal reads over the stored codes ----
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_buf = pm.data if pm.data.numel() * pm.data.element_size() >= (1 << 28) else torch.empty(1 << 28, dtype=torch.int32, device=dev).random_()
    for _ in range(3):
        twa.probe_read(probe_buf, sink)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(20):
        twa.probe_read(probe_buf, sink)
    c1.record()
    torch.cuda.synchronize()
    read_ceiling = 20 * probe_buf.numel() * probe_buf.element_size() / (c0.elapsed_time(c1) * 1e-3) / 1e9
    roofline["measured_read_ceiling_GBps"] = round(read_ceiling, 1)
    roofline["frac_of_measured_read_ceiling"] = round(achieved / read_ceiling, 4)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same stored P ---------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import twa_oracle as orc
        from oracle.bridge import to_oracle

        g_h = ring[0].cpu().numpy().astype(np.float64)
        w_h = w.cpu().numpy().astype(np.float64)
        off_h = plan.layer_off.cpu().numpy() if layerwise else None

        def oracle_step(cols):
            po = to_oracle(pm, cols=cols, layer_off=off_h)
            t = time.perf_counter()
            if layerwise:
                so = orc.project_layers(po, g_h, off_h)
                bo = np.zeros_like(so)
                orc.beta_step(bo, so, lr, lam)
                orc.weights_from_beta(po, bo, off_h, w_h)
            else:
                so = orc.project(po, g_h)
                orc.expand_update(po, so, w_h.copy(), lr)
            return time.perf_counter() - t

        t_one = oracle_step([0])
        m = int(max(1, min(n, round(args.cpu_seconds / max(t_one, 1e-6)))))
        reps, t_sum = 0, 0.0
        while reps == 0 or (m == n and t_sum < args.cpu_seconds and reps < 50):
            t_sum += oracle_step(list(range(m))) if m > 1 else oracle_step([0])
            reps += 1
        t_m = t_sum / reps
        cpu = {"value": round(1.0 / (t_m * n / m), 5), "unit": "steps/s", "cores": orc.threads(), "kind": "oracle",
               "sample": f"{reps} full step(s) ({'coefficient step + weights from coefficients, layer-wise' if layerwise else 'project + expand_update'}, fp64, on-the-fly dequantisation) over the "
                         f"first {m} of {n} basis vectors at full D={D}: {t_m:.2f} s per step-sample, scaled by {n}/{m}"}

    out = {
        "metric": METRIC if not layerwise else METRIC_LAYERWISE, "value": round(steps_per_s, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: D={D}, n={n}, P stored as {args.storage}"
                               + (f" (block {pm.block}, {'fp32' if dtype == twa.I8 else 'fp16'} scales)"
                                  if dtype in (twa.I8, twa.I4) else "")
                               + (f"; layer-wise, L={plan.L}, centre+normalise basis, coefficient form, lambda={lam}"
                                  if layerwise else ""),
                   "lr": lr, "sigma_g": wl.sigma_g, "gradient_ring": 4, "seed": args.seed},
        "p_stream_GBps": round(p_stream_gbps, 1), "p_stream_pct_of_peak": round(100 * p_stream_gbps / HBM_PEAK_GBPS, 2),
        "p_bytes_per_pass": p_bytes, "roofline": roofline, "cpu_baseline": cpu,
        "setup_s": {"generate": round(t1 - t0, 3), "build_basis": round(t2 - t1, 4), "quantize": round(t3 - t2, 4)},
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
