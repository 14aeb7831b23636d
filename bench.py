#!/usr/bin/env python3
"""Benchmark of the TWA projected-gradient step on one MI355X.

One "step" is one pass of the whole hot path over one synthetic gradient:
    s = P^T g   (twa_project)      then      g~ = P s, w -= lr g~   (twa_expand_update)
enqueued back to back on one stream, s staying on the device.  The default workload is the
ResNet-50-sized configuration the metric is quoted on: D = 25,557,032, n = 100, P stored as int8
codes with one fp32 absmax scale per 128 elements.  P is produced by the library itself from a
synthetic checkpoint trajectory (twa_build_basis, then twa_quantize); all inputs are resident in
HBM before the timed region starts.

Protocol: W untimed warm-up steps; K steps timed at once (the "cold" figure: what a short run sees
while the device's clocks still settle); further untimed steps until the device has been under this
load for --settle-seconds; then --reps repetitions of exactly K timed steps each, bracketed by
synchronisations.  `ms_per_step` and `value` are the MEDIAN repetition; the line keeps every
repetition and the cold figure.

Prints ONE JSON line.  `value` = projected steps/s; `p_stream_GBps` = steps/s x 2 x (bytes of P);
`roofline` = the slower of the two kernels against the 8 TB/s HBM peak, its duration measured here
with device events on the stream the kernels run on; `cpu_baseline` = the fp64 oracle timed on the
host cores (all of them, and one) on a bounded sample of the same stored P.

Other legs: --mode layerwise (Alg. 1 as written), --mode batched (s = P^T G for k gradients per call,
the fine-tuning configuration's own metric: calls/s and GB/s over ALL bytes, P + G).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, published peak
# issue peak of the vector ALUs: 256 compute units x 4 SIMDs x 16 lanes x 2.4 GHz lane-instructions per second
VALU_PEAK_TLANE = 256 * 4 * 16 * 2.4e9 / 1e12
METRIC = "projected steps/s and P-stream HBM GB/s (% of peak), D=25.6M n=100 int8"
STORAGE_NAME = {"f32": "fp32", "bf16": "bf16", "i8": "int8", "i4": "int4", "mm16": "minmax16", "mm8": "minmax8",
                "mm4": "minmax4", "mm3": "minmax3", "mm2": "minmax2", "mm1": "minmax1"}
# vector-ALU lane-instructions per stored element of the step kernels (projection-like, expansion-like), from
# rocprofv3 --pmc SQ_INSTS_VALU (profiles/sq_counters_imagenet_resnet50_int4_int8.txt): the expansion on 4-bit codes
# is co-limited by the vector ALUs; the projection on them computes in integer dot products and is not
VALU_INSTR_PER_ELEMENT = {"i8": (2.14, 2.28), "mm8": (2.14, 2.28), "i4": (1.67, 2.64), "mm4": (1.66, 2.53)}

def log(*a):
    print(*a, file=sys.stderr, flush=True)


def read_traffic(tag: str, kernel: str):
    """HBM bytes per launch measured with rocprofv3 --pmc for THIS leg, workload and storage
    (profiles/hbm_traffic_<tag>.txt), or None when no such measurement is committed."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}.txt")
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
    ap.add_argument("--steps", type=int, default=1000, help="K: steps per timed repetition")
    ap.add_argument("--warmup", type=int, default=200, help="W: untimed steps before anything is timed")
    ap.add_argument("--reps", type=int, default=5, help="timed repetitions of K steps; the median is reported")
    ap.add_argument("--settle-seconds", type=float, default=1.0,
                    help="the device runs this load for at least so long before the repetitions are timed "
                         "(its step time settles after ~0.5 s of load)")
    ap.add_argument("--workload", default="imagenet_resnet50", help="name in synth.WORKLOADS")
    ap.add_argument("--storage", default=None, choices=list(STORAGE_NAME),
                    help="mm16 .. mm1: the paper's per-layer min-max codes of that many bits (layer-wise mode only); "
                         "default: i8 (bf16 in batched mode)")
    ap.add_argument("--mode", default="whole", choices=["whole", "layerwise", "batched"],
                    help="whole: the headline step (orthonormal basis, s = P^T g, w -= lr P s).  layerwise: Alg. 1 as "
                         "written -- per-layer centre+normalise basis, coefficient step with weight decay, w = wbar + P beta.  "
                         "batched: projection only, k gradients per call (S = P^T G)")
    ap.add_argument("--batched", action="store_true", help="same as --mode batched")
    ap.add_argument("--k", type=int, default=0, help="gradients per call in batched mode (default: the workload's, 8)")
    ap.add_argument("--D", type=int, default=0, help="override the parameter count (smoke runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="target CPU time of each oracle sample")
    ap.add_argument("--basis-baseline", action="store_true",
                    help="also time the one-time basis construction: twa_build_basis on the device against the oracle's "
                         "Householder factorisation on the host cores, the latter on a slice of D rows and scaled (its cost is linear in D)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known 1 GiB read + 1 GiB write) so that a "
                         "rocprofv3 --pmc run of this command can scale FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is a single-GPU library (no collectives, no sharding); run with --gpus 1. "
                 "(It would shard by rows of P: every GPU holds a slice of all n vectors and of w, and one all-reduce of n floats per step joins the partial coefficients.)")
    if args.batched:
        args.mode = "batched"
    if args.storage is None:
        args.storage = "bf16" if args.mode == "batched" else "i8"

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
    batched = args.mode == "batched"
    if dtype in twa.MINMAX_TYPES and not layerwise:
        sys.exit("bench.py: the min-max formats exist for the layer-wise calls only (use --mode layerwise)")
    k = (args.k or max(wl.k, 2)) if batched else 1

    # ---- inputs: checkpoints -> orthonormal basis (in place) -> stored P ------------------------
    t0 = time.time()
    plan = None
    from_panels = wl.name == "large" and not layerwise and dtype in (twa.I8, twa.I4, twa.BF16) and D % 4 == 0
    if from_panels:
        # this configuration's checkpoints (179 GB in fp32) and its fp32 basis are never held: rows are produced in
        # panels of 2^24 into one staging buffer, three sweeps, the second pass fused with the quantiser
        from paper_2205_13104_amd.panels import stored_basis_from_panels
        w = torch.empty(D, dtype=torch.float32, device=dev)

        def make_panel(r0, rows, stage):
            synth.trajectory_panel(rows, n, wl.decay, wl.drift, args.seed, r0, stage)

        def mean_of(r0, rows, stage):                       # the plain average: starting point of TWA
            w[r0:r0 + rows] = stage[:, :rows].mean(dim=0)

        t1 = time.time()
        outs, _, _, stage, _ = stored_basis_from_panels(make_panel, D, n, 1 << 24, [dtype], device=dev, on_first_sweep=mean_of)
        pm = outs[dtype]
        torch.cuda.synchronize()
        t2 = t3 = time.time()
        del stage, outs
        torch.cuda.empty_cache()
        log(f"[bench] {wl.name}: D={D} n={n} storage={args.storage} mode={args.mode}; basis and stored matrix from "
            f"panels of 2^24 rows in {t2 - t1:.2f}s (generation included); peak device memory "
            f"{torch.cuda.max_memory_allocated() / 2**30:.1f} GiB")
    else:
        W = synth.checkpoints(wl, seed=args.seed, device=dev, D=D)
        w = W[:, :D].mean(dim=0).contiguous()                  # the plain average: starting point of TWA
        torch.cuda.synchronize()
        t1 = time.time()
        if layerwise:
            sizes = synth.workload_layers(wl.name) if D == wl.D else synth.layer_offsets(synth.random_layer_sizes(D, 12, 11))
            plan = twa.LayerPlan(sizes, D)
            P32, w, _ = twa.centre_normalise(W, D, plan, out=W, want_norms=False)     # w = wbar: Alg. 1 starts at the mean
            wbar = w.clone()
        elif wl.name == "large":
            P32, _ = twa.build_basis_panels(W, D, 1 << 24, out=W)      # (fp32 storage: the panels are views of W)
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
        log(f"[bench] {wl.name}: D={D} n={n} storage={args.storage} mode={args.mode}; generate {t1 - t0:.2f}s, "
            f"build_basis {t2 - t1:.3f}s, quantize {t3 - t2:.3f}s")
    if args.calibrate_copy:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        b = torch.empty_like(a)
        torch.cuda.synchronize()
        b.copy_(a)                                   # the calibration kernel: reads 2^30 B, writes 2^30 B
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()
    lr = wl.lr
    lam = 1e-4                                  # weight decay of the coefficient form (layer-wise mode)
    p_bytes = pm.stream_bytes
    if batched:
        ldg = (D + 3) // 4 * 4
        nring = 2                               # a batch of gradients is far larger than every cache of the device
        ring = [synth.gradient(D, wl.sigma_g, seed=args.seed, step=i, device=dev, k=k, ldg=ldg) for i in range(nring)]
        S = torch.empty((k, n), dtype=torch.float32, device=dev)
        ws = twa.Workspace(twa.project_workspace_bytes(n, k), device=dev)

        def step(i):
            twa.project(pm, ring[i % nring], S, ws)

        legs = {"twa_project": (lambda i: twa.project(pm, ring[i % nring], S, ws), p_bytes + 4 * D * k + 4 * n * k)}
        pass_per_step, unit = 1, "calls/s"
    elif layerwise:
        nring = 4
        ring = [synth.gradient(D, wl.sigma_g, seed=args.seed, step=i, device=dev) for i in range(nring)]
        L = plan.L
        beta = torch.zeros((L, n), dtype=torch.float32, device=dev)
        ws = twa.Workspace(twa.project_layers_workspace_bytes(n, L), device=dev)

        def step(i):
            twa.beta_step(pm, ring[i & 3], plan, beta, lr, lam, None, ws)
            twa.weights_from_beta(pm, beta, plan, wbar, w)

        legs = {
            # P once + g + beta read and written
            "twa_beta_step": (lambda i: twa.beta_step(pm, ring[i & 3], plan, beta, lr, lam, None, ws), p_bytes + 4 * D + 8 * n * L),
            # P once + wbar read + w written + beta
            "twa_weights_from_beta": (lambda i: twa.weights_from_beta(pm, beta, plan, wbar, w), p_bytes + 8 * D + 4 * n * L),
        }
        pass_per_step, unit = 2, "steps/s"
    else:
        nring = 4
        ring = [synth.gradient(D, wl.sigma_g, seed=args.seed, step=i, device=dev) for i in range(nring)]
        s = torch.empty(n, dtype=torch.float32, device=dev)
        ws = twa.Workspace(twa.project_workspace_bytes(n), device=dev)

        def step(i):
            twa.project(pm, ring[i & 3], s, ws)
            twa.expand_update(pm, s, w, lr)

        legs = {
            "twa_project": (lambda i: twa.project(pm, ring[i & 3], s, ws), p_bytes + 4 * D + 4 * n),            # P once + g + s
            "twa_expand_update": (lambda i: twa.expand_update(pm, s, w, lr), p_bytes + 8 * D + 4 * n),        # P once + w read + w write + s
        }
        pass_per_step, unit = 2, "steps/s"

    def timed_steps(count):
        """`count` steps between two device events on the kernels' stream and two host clock readings, both
        bracketed by synchronisations; the larger of the two times, in ms."""
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        wall0 = time.perf_counter()
        e0.record()
        for i in range(count):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - wall0
        return max(e0.elapsed_time(e1), wall * 1e3)

    # ---- warm-up, the cold figure, settling, then the timed repetitions of exactly K steps ----------
    K = args.steps
    load0 = time.perf_counter()
    for i in range(args.warmup):
        step(i)
    cold_ms = timed_steps(K) / K                         # what a single short run would report
    settle_steps = 0
    while time.perf_counter() - load0 < args.settle_seconds:
        for i in range(32):
            step(i)
        settle_steps += 32
        torch.cuda.synchronize()
    load_s = time.perf_counter() - load0
    rep_ms = [timed_steps(K) / K for _ in range(max(1, args.reps))]
    ms_per_step = statistics.median(rep_ms)
    steps_per_s = 1e3 / ms_per_step
    p_stream_gbps = steps_per_s * pass_per_step * p_bytes / 1e9

    # ---- launch-bound workloads: the same K steps captured once in a HIP graph and replayed ----------
    graph_ms = None
    if ms_per_step < 0.1 and K <= 4096:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for i in range(8):
                step(i)                                      # warm-up on the capture stream
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            for i in range(K):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        reps_g = []
        for _ in range(max(1, args.reps)):
            g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            wall0 = time.perf_counter()
            g0.record()
            graph.replay()
            g1.record()
            torch.cuda.synchronize()
            reps_g.append(max(g0.elapsed_time(g1), (time.perf_counter() - wall0) * 1e3) / K)
        graph_ms = statistics.median(reps_g)

    # ---- per-kernel launch durations (device events around every launch, same stream) ----------
    K2 = max(20, min(K, 200))

    def timed_each(fn):
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K2)]
        for i, (a, b) in enumerate(evs):
            a.record()
            fn(i)
            b.record()
        torch.cuda.synchronize()
        return statistics.median(a.elapsed_time(b) for a, b in evs)

    dur = {name: timed_each(fn) for name, (fn, _) in legs.items()}
    alg = {name: nbytes for name, (_, nbytes) in legs.items()}
    dom = max(dur, key=dur.get)
    achieved = alg[dom] / (dur[dom] * 1e-3) / 1e9
    tag = ("layerwise_" if layerwise else "batched_" if batched else "") + f"{wl.name}_{STORAGE_NAME[args.storage]}"
    roofline = {"bound": "hbm", "kernel": dom, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4),
                "traffic": read_traffic(tag, dom) if D == wl.D else None,
                "algorithmic_bytes_per_launch": alg[dom], "avg_launch_ms": round(dur[dom], 5)}
    others = [nm for nm in dur if nm != dom]
    if others:
        o = others[0]
        roofline["other_kernel"] = {"kernel": o, "avg_launch_ms": round(dur[o], 5),
                                    "achieved": round(alg[o] / (dur[o] * 1e-3) / 1e9, 1)}
    if args.storage in VALU_INSTR_PER_ELEMENT:
        # the second bound of the integer-code kernels: vector-ALU issue (decode + FMA per stored element)
        per_elem = VALU_INSTR_PER_ELEMENT[args.storage][0 if ("project" in dom or "beta_step" in dom) else 1]
        lane_instr = per_elem * n * D
        tl = lane_instr / (dur[dom] * 1e-3) / 1e12
        roofline["valu"] = {"lane_instr_per_element": per_elem,
                            "achieved_Tlane_instr_per_s": round(tl, 2), "peak": round(VALU_PEAK_TLANE, 2),
                            "frac": round(tl / VALU_PEAK_TLANE, 4),
                            "note": "co-limited: neither HBM nor the vector ALUs saturated" if tl / VALU_PEAK_TLANE > 0.5
                            else "HBM bound; the vector ALUs are mostly idle"}

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

        g_h = (ring[0][:, :D] if batched else ring[0]).cpu().numpy().astype(np.float64)
        w_h = w.cpu().numpy().astype(np.float64)
        off_h = plan.layer_off.cpu().numpy() if layerwise else None
        what = ("coefficient step + weights from coefficients, layer-wise" if layerwise
                else f"projection of {k} gradients" if batched else "project + expand_update")

        def oracle_step(cols):
            po = to_oracle(pm, cols=cols, layer_off=off_h)
            t = time.perf_counter()
            if layerwise:
                so = orc.project_layers(po, g_h, off_h)
                bo = np.zeros_like(so)
                orc.beta_step(bo, so, lr, lam)
                orc.weights_from_beta(po, bo, off_h, w_h)
            elif batched:
                orc.project(po, g_h)
            else:
                so = orc.project(po, g_h)
                orc.expand_update(po, so, w_h.copy(), lr)
            return time.perf_counter() - t

        def sample(budget_s):
            """Steps/s of the oracle from a sample of about `budget_s` seconds: whole steps if one fits the budget,
            else one step over the first m basis vectors, scaled by n/m (both passes are linear in the vectors)."""
            t_one = oracle_step([0])
            m = int(max(1, min(n, round(budget_s / max(t_one, 1e-6)))))
            reps, t_sum = 0, 0.0
            while reps == 0 or (m == n and t_sum < budget_s and reps < 50):
                t_sum += oracle_step(list(range(m)))
                reps += 1
            t_m = t_sum / reps
            return 1.0 / (t_m * n / m), f"{reps} step(s) over the first {m} of {n} basis vectors at full D={D}: {t_m:.2f} s each, scaled by {n}/{m}"

        all_cores = orc.threads()
        v_all, how_all = sample(args.cpu_seconds)
        orc.set_threads(1)
        v_one, how_one = sample(args.cpu_seconds * 0.75)
        orc.set_threads(all_cores)
        cpu = {"value": round(v_all, 5), "unit": unit, "cores": all_cores, "kind": "oracle",
               "sample": f"{what}, fp64, on-the-fly dequantisation; {how_all}",
               "one_core": {"value": round(v_one, 5), "unit": unit, "cores": 1, "sample": how_one}}

    # ---- the one-time basis construction against the oracle's (optional leg) ---------------------------
    basis = None
    if args.basis_baseline and not from_panels:
        from oracle import twa_oracle as orc
        Wb = synth.checkpoints(wl, seed=args.seed, device=dev, D=D)
        Pb = torch.empty_like(Wb)
        wsb = twa.Workspace(twa.build_basis_workspace_bytes(n), device=dev)
        twa.build_basis(Wb, D, out=Pb, want_R=False, ws=wsb)
        torch.cuda.synchronize()
        tb = []
        for _ in range(5):
            t = time.perf_counter()
            twa.build_basis(Wb, D, out=Pb, want_R=False, ws=wsb)
            torch.cuda.synchronize()
            tb.append(time.perf_counter() - t)
        Ds = max(4 * n, min(D, 1_000_000))
        Wh = Wb[:, :Ds].cpu().numpy().astype(np.float64)
        del Wb, Pb
        t = time.perf_counter()
        orc.build_basis(Wh)
        t_or = time.perf_counter() - t
        basis = {"twa_build_basis_ms": round(1e3 * statistics.median(tb), 3),
                 "oracle_s": round(t_or * D / Ds, 2), "cores": orc.threads(),
                 "sample": f"Householder QR in fp64 of the first {Ds} of {D} rows of the same {n} checkpoints: {t_or:.2f} s, scaled by {D}/{Ds}"}

    store_txt = f"P stored as {args.storage}" + (f" (block {pm.block}, {'fp32' if dtype == twa.I8 else 'fp16'} scales)"
                                                  if dtype in (twa.I8, twa.I4) else "")
    headline = (args.mode == "whole" and wl.name == "imagenet_resnet50" and args.storage == "i8" and D == wl.D)
    if headline:
        metric = METRIC
    elif batched:
        metric = f"batched projections/s (k={k} gradients per call) and HBM GB/s over all bytes (% of peak), {wl.name} D={D} n={n} {args.storage}"
    elif layerwise:
        metric = f"layer-wise coefficient-form steps/s (Alg. 1) and P-stream HBM GB/s (% of peak), {wl.name} D={D} n={n} {args.storage}"
    else:
        metric = f"projected steps/s and P-stream HBM GB/s (% of peak), {wl.name} D={D} n={n} {args.storage}"
    out = {
        "metric": metric, "value": round(steps_per_s, 2), "unit": unit, "n_gpus": 1, "steps": K,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: D={D}, n={n}, {store_txt}"
                               + (f"; layer-wise, L={plan.L}, centre+normalise basis, coefficient form, lambda={lam}" if layerwise else "")
                               + (f"; projection only, k={k} gradients per call" if batched else ""),
                   "lr": lr, "sigma_g": wl.sigma_g, "gradient_ring": nring, "seed": args.seed},
        "timing": {"protocol": f"median of {len(rep_ms)} repetitions of {K} steps after {args.warmup} warm-up steps and "
                               f"{load_s:.2f} s of this load on the device",
                   "rep_ms_per_step": [round(x, 5) for x in rep_ms], "min_ms_per_step": round(min(rep_ms), 5),
                   "max_ms_per_step": round(max(rep_ms), 5), "cold_ms_per_step": round(cold_ms, 5),
                   "cold_note": f"the {K} steps right after the {args.warmup} warm-up steps, before the device's step time has settled",
                   "settle_steps": settle_steps, "device_load_s_before_timing": round(load_s, 3)},
        "p_stream_GBps": round(p_stream_gbps, 1), "p_stream_pct_of_peak": round(100 * p_stream_gbps / HBM_PEAK_GBPS, 2),
        "p_bytes_per_pass": p_bytes, "roofline": roofline, "cpu_baseline": cpu,
        "setup_s": {"generate": round(t1 - t0, 3), "build_basis": round(t2 - t1, 4), "quantize": round(t3 - t2, 4)},
    }
    if basis is not None:
        out["basis_construction"] = basis
    if graph_ms is not None:
        out["hip_graph"] = {"ms_per_step": round(graph_ms, 5), "steps_per_s": round(1e3 / graph_ms, 1),
                            "note": f"the same {K} steps captured once in a HIP graph and replayed (median of {max(1, args.reps)}): "
                                    "this workload is bound by launches, not by bytes"}
    if batched:
        tot = alg["twa_project"]
        out["total_GBps"] = round(steps_per_s * tot / 1e9, 1)
        out["total_pct_of_peak"] = round(100 * steps_per_s * tot / 1e9 / HBM_PEAK_GBPS, 2)
        out["total_bytes_per_call"] = tot
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
