#!/usr/bin/env python3
"""Benchmark of the TensorGRaD optimizer hot path on one MI355X.

One "step" = one `tgrad_step` on one synthetic FNO-shaped gradient already resident in HBM
(refresh of support and factors included whenever t % T == 0 falls in the timed region).
Prints ONE JSON line: whole-job throughput in Gelem/s, the roofline of the dominant kernel
(per-kernel durations from HIP events recorded by the library on its own stream), and the CPU
oracle timed on a bounded sample of the same workload.
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

import numpy as np

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_FP32_PEAK_TF = 157.3      # dense fp32 matrix
MFMA_FP64_PEAK_TF = 78.6       # dense fp64 matrix


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def kernel_model(w, fused, weight_bytes=8, core_fused=0):
    """Algorithmic bytes and flops per launch of every kernel, from the tensor shapes alone
    (8 real flops per complex multiply-add; a complex64 element is 8 bytes).  `fused`: the library
    ran the mode-(N-1) compression / reconstruction stages inside the first-stage and the
    weight-update kernels (it does whenever the shape allows), so the tensors between them are
    neither written nor read.  `weight_bytes`: 8 for complex64 weights, 4 for bf16 pairs.
    `core_fused`: how many leading modes the kernel around the core handles both ways (0, 1 or 2)."""
    shape, ranks, k = w.shape, w.ranks, w.k
    N = len(shape)
    I = int(np.prod(shape))
    C = int(np.prod(ranks))
    gb = 8 if w.grad_dtype == "c64" else 4
    m = {}

    def stage_dims(project, s):
        if project:
            n = N - 1 - s
            A = int(np.prod(shape[:n])) if n else 1
            B = int(np.prod(ranks[n + 1:])) if n + 1 < N else 1
            return A, shape[n], ranks[n], B
        n = s
        A = int(np.prod(shape[:n])) if n else 1
        B = int(np.prod(ranks[n + 1:])) if n + 1 < N else 1
        return A, ranks[n], shape[n], B

    def vol(A, K, M, B):
        return (A * K * B + A * M * B) * 8, 8 * A * K * M * B

    # first compression stage (contracts the last mode of G itself) fused with the sparse gather
    A, K, M, B = stage_dims(True, 0)
    by, fl = I * gb + A * M * B * 8 + k * (4 + 8), 8 * A * K * M * B
    first_mid = 1
    if fused:
        A1, K1, M1, B1 = stage_dims(True, 1)
        by += A1 * M1 * B1 * 8 - A * M * B * 8             # writes the stage-1 result instead of its own
        fl += 8 * A1 * K1 * M1 * B1
        first_mid = 2
    m["project_first"] = {"bytes": by, "flops": fl, "bound": "hbm"}
    # `core_fused`: the last 1 or 2 compression stages, AdamUpdate on the core and the first 1 or 2
    # reconstruction stages run as one kernel: reads its input tensor, writes a tensor of the
    # same size, reads and writes the moments and writes the core gradient
    proj_end = N - core_fused
    by = fl = 0
    for s in range(first_mid, proj_end):
        b_, f_ = vol(*stage_dims(True, s))
        by += b_
        fl += f_
    if proj_end > first_mid:
        m["project"] = {"bytes": by, "flops": fl, "bound": "mfma", "launches_per_step": proj_end - first_mid}
    last_mid = N - 2 if fused else N - 1                  # reconstruction stages 0 .. last_mid - 1 run alone
    back_start = core_fused
    by = fl = 0
    for s in range(back_start, last_mid):
        b_, f_ = vol(*stage_dims(False, s))
        by += b_
        fl += f_
    if last_mid > back_start:
        m["backproject"] = {"bytes": by, "flops": fl, "bound": "mfma", "launches_per_step": last_mid - back_start}
    if core_fused:
        A0, K0, M0, B0 = stage_dims(True, N - core_fused)    # the kernel's input: (A0, K0, B0), A0 = I_1 with two modes
        fl = sum(2 * vol(*stage_dims(True, s))[1] for s in range(N - core_fused, N))
        m["core"] = {"bytes": 2 * A0 * K0 * B0 * 8 + C * (8 + 12 + 12), "flops": fl + 12 * C, "bound": "mfma"}
    # last reconstruction stage fused with the sparse AdamUpdate, the scatter-add and the weight
    # update: reads its input tensor and W, writes W; per sparse entry its index, gathered value
    # and both moments are read and the moments written back
    A, K, M, B = stage_dims(False, N - 1)
    by, fl = A * K * 8 + 2 * weight_bytes * I + k * (4 + 8 + 12 + 12), 8 * A * K * M + 4 * I + 14 * k
    if fused:
        A1, K1, M1, B1 = stage_dims(False, N - 2)
        by += A1 * K1 * B1 * 8 - A * K * 8                  # reads the stage-(N-2) input instead
        fl += 8 * A1 * K1 * M1 * B1
    m["update"] = {"bytes": by, "flops": fl, "bound": "hbm"}
    m["gather"] = {"bytes": k * (4 + gb + 8), "flops": 0, "bound": "hbm"}
    m["adam_core"] = {"bytes": C * (8 + 12 + 12 + 8), "flops": 12 * C, "bound": "hbm"}
    m["sparse_update"] = {"bytes": k * (8 + 4 + 12 + 12 + 16), "flops": 14 * k, "bound": "hbm"}
    # selection: two streaming reads of G (leading-digit histogram; the pass that writes the two
    # bitmasks, I/8 bytes each); the later kernels read the masks and the candidates' keys only
    m["select_hist"] = {"bytes": I * gb, "flops": 3 * I, "bound": "hbm"}
    m["select_split"] = {"bytes": I * gb + 2 * (I // 8), "flops": 3 * I, "bound": "hbm"}
    m["select_count"] = {"bytes": 2 * (I // 8), "flops": 0, "bound": "hbm"}
    m["select_emit"] = {"bytes": 3 * (I // 8) + 4 * k, "flops": 0, "bound": "hbm"}
    # a Gram matrix is Hermitian: I (I_n + 1) / 2 complex multiply-adds give all of it
    gram_fl = sum(8 * I * (shape[n] + 1) // 2 for n in range(N) if ranks[n] < shape[n])
    ngram = sum(1 for n in range(N) if ranks[n] < shape[n])
    m["gram"] = {"bytes": ngram * I * gb, "flops": gram_fl, "bound": "mfma64", "launches_per_step": ngram}
    return m


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel`, measured with rocprofv3 --pmc (FETCH_SIZE and WRITE_SIZE,
    scaled by the calibration copy) and recorded in the text summary under profiles/; None when no
    such measurement is recorded for this workload."""
    import re
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s.txt" % workload)
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"^%s\s+traffic_bytes_per_launch\s*=\s*(\d+)" % re.escape(kernel), text, flags=re.M)
    return int(m.group(1)) if m else None


def cpu_baseline(w):
    """The oracle, as it stands, on the workload itself: the gradient of layer 0 from the same
    seeded generator the GPU run uses, one refresh + 3 steps (the steps after the first run on the
    old support), amortised over the workload's refresh period exactly like the GPU figure.  A
    workload of several layers is timed on one layer (every layer costs the same)."""
    from oracle import tgrad_oracle as O
    from paper_2501_02379_amd import synth
    I = w.numel
    grads = [synth.gradient(w, t) for t in range(2)]
    st = O.State(w.shape, O.Hyper(ranks=w.ranks, k=w.k, lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                                  alpha=w.alpha, lam=w.lam, weight_decay=w.weight_decay, T=0))
    W = synth.initial_weight(w).astype(np.complex128)
    t0 = time.perf_counter()
    O.refresh(st, grads[0])
    t_refresh = time.perf_counter() - t0
    nsteps = 3
    t0 = time.perf_counter()
    for t in range(nsteps):
        W = O.step(st, W, grads[t & 1])
    t_step = (time.perf_counter() - t0) / nsteps
    per_step = t_step + t_refresh / max(1, w.T)
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas = None
    return {
        "value": I / per_step / 1e9, "unit": "Gelem/s", "cores": int(cores), "blas_threads": blas, "kind": "oracle",
        "sample": "the %s gradient itself (%s, %d elements, one layer), ranks %s, k=%d; 1 refresh (%.2f s) + %d "
                  "steps (%.2f s each), amortised over T=%d" % (w.name, "x".join(map(str, w.shape)), I,
                                                               ",".join(map(str, w.ranks)), w.k, t_refresh, nsteps,
                                                               t_step, w.T),
        "refresh_s": round(t_refresh, 3), "step_s": round(t_step, 3),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=20,
                    help="untimed steps first (the clocks take some tens of steps to settle; step 0 refreshes)")
    ap.add_argument("--workload", default="cfg4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--probe-copies", type=int, default=50,
                    help="launches of the copy kernel that measure the achievable HBM rate (they run right before the timed steps)")
    ap.add_argument("--hooi-sweeps", type=int, default=0,
                    help="HOOI refinement sweeps per refresh (default 0 = HOSVD factors, the headline configuration)")
    ap.add_argument("--warm-restart", action="store_true", help="with --hooi-sweeps: refreshes restart from the factors in place")
    ap.add_argument("--select", choices=("topk", "random"), default="topk",
                    help="support selection rule (default top-k magnitude, the headline configuration)")
    ap.add_argument("--order", choices=("us_lr", "lr_us", "sum"), default="us_lr",
                    help="composition of the two components (default us_lr = Algorithm 1, the headline configuration)")
    ap.add_argument("--weights", choices=("c64", "bf16"), default="c64",
                    help="weight storage (default complex64, the headline configuration; bf16 = half-precision pairs)")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (one process, one MI355X); --gpus %d is not supported."
            % args.gpus)
        sys.exit(2)

    import torch
    from paper_2501_02379_amd import synth, tgrad as T

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(2)
    T.load()                                    # raises if the HIP library is not built
    w = synth.WORKLOADS[args.workload]
    K = args.steps if args.steps is not None else w.T
    Wm = args.warmup
    dev = "cuda:0"
    I = w.numel * w.layers

    log("generating inputs for %s %s ..." % (w.name, "x".join(map(str, w.shape))))
    ctxs, Ws, Gs = [], [], []
    for layer in range(w.layers):
        cfg = T.make_config(w.shape, w.ranks, w.k, grad_dtype=T.TGRAD_CBF16 if w.grad_dtype == "cbf16" else 0,
                            lr=w.lr, beta1=w.beta1, beta2=w.beta2, eps=w.eps, alpha=w.alpha, lam=w.lam,
                            weight_decay=w.weight_decay, refresh_every=w.T, hooi_sweeps=args.hooi_sweeps,
                            warm_restart=args.warm_restart,
                            select_rule=T.TGRAD_SELECT_RANDOM if args.select == "random" else T.TGRAD_SELECT_TOPK_MAG,
                            select_seed=2501 + layer,
                            order={"us_lr": T.TGRAD_ORDER_US_LR, "lr_us": T.TGRAD_ORDER_LR_US, "sum": T.TGRAD_ORDER_SUM}[args.order],
                            weight_dtype=T.TGRAD_CBF16 if args.weights == "bf16" else T.TGRAD_C64)
        ctxs.append(T.Context(cfg, device=dev))
        w0 = synth.initial_weight(w, layer)
        Ws.append(T.to_device_weight(synth.complex64_to_bf16_pairs(w0) if args.weights == "bf16" else w0, dev))
        Gs.append([T.to_device_grad(synth.gradient(w, t, layer), dev) for t in range(2)])
    torch.cuda.synchronize()

    def run_steps(n, t0):
        for t in range(t0, t0 + n):
            for layer in range(w.layers):
                ctxs[layer].tgrad_step(Ws[layer], Gs[layer][t & 1])

    log("warmup %d steps ..." % Wm)
    run_steps(Wm, 0)
    torch.cuda.synchronize()

    # ---- achievable HBM rate on this machine, in this run: the library's plain copy kernel on a
    # gradient-sized buffer (bytes read + bytes written over the HIP-event time)
    nb = w.numel * 8 // 16 * 16          # (also the known-size launch that scales the profiler's HBM counters)
    csrc = torch.empty(nb, dtype=torch.uint8, device=dev)
    cdst = torch.empty_like(csrc)
    csrc.zero_()
    ce0, ce1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        T.tgrad_calibration_copy(cdst, csrc)
    ncopy = max(1, args.probe_copies)
    ce0.record()
    for _ in range(ncopy):
        T.tgrad_calibration_copy(cdst, csrc)
    ce1.record()
    torch.cuda.synchronize()
    copy_gbs = 2.0 * nb * ncopy / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    # ... and what the memory system gives the weight-update kernel's own access pattern (one tile of 32 rows
    # of the last mode per wavefront, loaded whole and stored back in place; slabs of I_(N-1) / 32 tiles)
    tile_bytes = 32 * w.shape[-1] * 8
    tile_gbs = None
    if len(w.shape) >= 2 and tile_bytes <= 17 * 1024 and w.shape[-2] % 32 == 0:
        for _ in range(2):
            T.tgrad_calibration_tile_stream(cdst, tile_bytes, w.shape[-2] // 32)
        ce0.record()
        moved = 0
        for _ in range(10):
            moved += T.tgrad_calibration_tile_stream(cdst, tile_bytes, w.shape[-2] // 32)
        ce1.record()
        torch.cuda.synchronize()
        tile_gbs = 2.0 * moved / (ce0.elapsed_time(ce1) * 1e-3) / 1e9
    del csrc, cdst

    # ---- region A: the timed K steps (no per-kernel events) ----
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    run_steps(K, Wm)
    e1.record()
    torch.cuda.synchronize()
    ms_total = e0.elapsed_time(e1)
    ms_per_step = ms_total / K
    refreshes = sum(1 for t in range(Wm, Wm + K) if t % w.T == 0)
    value = I / (ms_per_step * 1e-3) / 1e9

    # ---- region B: the same K steps again with per-kernel HIP events on the library's stream ----
    for c in ctxs:
        c.tgrad_set_profiling(True)
    torch.cuda.synchronize()
    e0.record()
    run_steps(K, Wm + K)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step_profiled = e0.elapsed_time(e1) / K
    times = {}
    for c in ctxs:
        for name, v in c.tgrad_get_kernel_times().items():
            d = times.setdefault(name, {"total_ms": 0.0, "launches": 0})
            d["total_ms"] += v["total_ms"]
            d["launches"] += v["launches"]
    # one explicit refresh, timed as a whole without events, then once more with per-kernel events so
    # that the refresh kernels are always covered
    for c in ctxs:
        c.tgrad_set_profiling(False)
    torch.cuda.synchronize()
    e0.record()
    for layer in range(w.layers):
        ctxs[layer].tgrad_refresh_factors(Gs[layer][0])
    e1.record()
    torch.cuda.synchronize()
    refresh_ms = e0.elapsed_time(e1)
    for c in ctxs:
        c.tgrad_set_profiling(True)
    for layer in range(w.layers):
        ctxs[layer].tgrad_refresh_factors(Gs[layer][0])
    torch.cuda.synchronize()
    rtimes = {}
    for c in ctxs:
        for name, v in c.tgrad_get_kernel_times().items():
            d = rtimes.setdefault(name, {"total_ms": 0.0, "launches": 0})
            d["total_ms"] += v["total_ms"]
            d["launches"] += v["launches"]
    times.update(rtimes)          # refresh kernels: the explicit refresh (step kernels never run in it)

    # ---- what the matrix cores deliver with nothing in the way, on this machine, in this run: the library's
    # register-resident loops of the float32 (projections) and float64 (Gram) matrix instructions (after
    # everything that is timed: the float64 loop draws enough power to lower the clocks for a while)
    sink = torch.zeros(4, dtype=torch.float32, device=dev)
    mfma_tf = {}
    for kind, key in ((0, "fp32"), (1, "fp64")):
        for _ in range(2):
            T.tgrad_calibration_mfma(kind, 4096, sink)
        ce0.record()
        fl = 0.0
        for _ in range(5):
            fl += T.tgrad_calibration_mfma(kind, 4096, sink)
        ce1.record()
        torch.cuda.synchronize()
        mfma_tf[key] = fl / (ce0.elapsed_time(ce1) * 1e-3) / 1e12


    # the library fuses the mode-(N-1) stages when the shape allows: then k_mid runs N - 2 times each way
    nstep = max(1, times.get("project_first", {}).get("launches", 1))
    # and the kernel around the core takes one leading mode, or two (four-way tensors, first extent 128):
    # the stages that k_mid does not launch are the ones that were absorbed
    nmid = times.get("project", {}).get("launches", 0) // nstep
    absorbed = (len(w.shape) - 1) - nmid - (1 if "core" in times else 0)
    fused = len(w.shape) >= 3 and absorbed >= 1
    core_fused = (2 if absorbed >= 2 else 1) if "core" in times else 0
    model = kernel_model(w, fused, 4 if args.weights == "bf16" else 8, core_fused)
    kernels = {}
    for name, v in sorted(times.items(), key=lambda kv: -kv[1]["total_ms"]):
        avg = v["total_ms"] / max(1, v["launches"])
        ent = {"avg_ms": round(avg, 5), "launches": v["launches"], "total_ms": round(v["total_ms"], 3)}
        mm = model.get(name)
        if mm:
            lp = mm.get("launches_per_step", 1)
            gbs = mm["bytes"] / lp / (avg * 1e-3) / 1e9
            tfl = mm["flops"] / lp / (avg * 1e-3) / 1e12
            ent["GBps"] = round(gbs, 1)
            ent["TFLOPs"] = round(tfl, 2)
            if mm["bound"] == "hbm":
                ent["frac_hbm_peak"] = round(gbs / HBM_PEAK_GBS, 4)
                ent["frac_hbm_achievable"] = round(gbs / copy_gbs, 4)
            elif mm["bound"] == "mfma64":
                ent["frac_mfma_fp64_peak"] = round(tfl / MFMA_FP64_PEAK_TF, 4)
                ent["frac_mfma_fp64_achievable"] = round(tfl / mfma_tf["fp64"], 4)
            else:
                ent["frac_mfma_fp32_peak"] = round(tfl / MFMA_FP32_PEAK_TF, 4)
                ent["frac_mfma_fp32_achievable"] = round(tfl / mfma_tf["fp32"], 4)
            if name == "project_first":          # straddles the ridge: both fractions
                ent["frac_mfma_fp32_peak"] = round(tfl / MFMA_FP32_PEAK_TF, 4)
                ent["frac_mfma_fp32_achievable"] = round(tfl / mfma_tf["fp32"], 4)
        kernels[name] = ent
    refresh_names = ("select", "gram", "eig", "mask", "factor", "hooi", "tile", "residual", "gather")
    step_kernels = [n for n in kernels if not n.startswith(refresh_names)]
    dom = max(step_kernels, key=lambda n: kernels[n]["total_ms"]) if step_kernels else None
    roofline = None
    if dom and dom in model:
        mm = model[dom]
        lp = mm.get("launches_per_step", 1)
        avg_s = kernels[dom]["avg_ms"] * 1e-3
        if mm["bound"] == "hbm":
            ach, peak, unit = mm["bytes"] / lp / avg_s / 1e9, HBM_PEAK_GBS, "GB/s"
        else:
            ach, peak, unit = mm["flops"] / lp / avg_s / 1e12, MFMA_FP32_PEAK_TF, "TFLOP/s"
        traffic = measured_traffic(w.name, dom) if args.weights == "c64" else None
        roofline = {"kernel": dom, "bound": "hbm" if mm["bound"] == "hbm" else "mfma",
                    "achieved": round(ach, 2), "peak": peak, "unit": unit, "frac": round(ach / peak, 4),
                    "traffic": traffic,
                    "traffic_source": ("profiles/hbm_traffic_%s.txt (rocprofv3 --pmc passes recorded earlier, not "
                                       "measured by this run)" % w.name) if traffic is not None else None,
                    "algorithmic_bytes_per_launch": mm["bytes"] // lp,
                    "avg_launch_ms": kernels[dom]["avg_ms"]}
        if mm["bound"] == "hbm":
            # what a plain copy kernel reaches on this machine in this run (read + write bytes per second)
            roofline["achievable_peak"] = round(copy_gbs, 1)
            roofline["frac_vs_achievable"] = round(ach / copy_gbs, 4)
            if dom == "update" and tile_gbs is not None and args.weights == "c64":
                # the same bytes moved with the update kernel's access pattern and no arithmetic
                roofline["pattern_ceiling"] = round(tile_gbs, 1)
                roofline["frac_vs_pattern_ceiling"] = round(ach / tile_gbs, 4)
    # selection as a whole: one read of G is what the method needs (8 or 4 bytes per element)
    sel_ms = sum(v["total_ms"] for n, v in rtimes.items() if n.startswith("select")) / max(1, w.layers)
    gbytes = w.numel * (8 if w.grad_dtype == "c64" else 4)
    select_summary = None
    if sel_ms > 0 and args.select == "topk":
        select_summary = {"ms_per_refresh": round(sel_ms, 4), "algorithmic_bytes": gbytes,
                          "GBps": round(gbytes / (sel_ms * 1e-3) / 1e9, 1),
                          "frac_hbm_peak": round(gbytes / (sel_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                          "frac_hbm_achievable": round(gbytes / (sel_ms * 1e-3) / 1e9 / copy_gbs, 4)}
    ms_amortised = None
    steady = ms_per_step if refreshes == 0 else None
    if refreshes == 0:
        ms_amortised = ms_per_step + refresh_ms / w.T
    elif K == w.T and refreshes == 1:
        ms_amortised = ms_per_step                      # exactly one period inside the timed region

    out = {
        "metric": "gradient elements compressed+updated/sec (Gelem/s) per step; % HBM roofline",
        "value": round(value, 4), "unit": "Gelem/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "%s: %d x %s %s gradient, Tucker ranks %s, k=%d sparse, refresh every %d"
                               % (w.name, w.layers, "x".join(map(str, w.shape)), w.grad_dtype,
                                  ",".join(map(str, w.ranks)), w.k, w.T),
                   "refreshes_in_timed_region": refreshes, "fused_mode_stages": bool(fused), "core_kernel_modes": int(core_fused),
                   "order": args.order, "weights": args.weights, "select": args.select, "hooi_sweeps": args.hooi_sweeps, "warm_restart": bool(args.warm_restart)},
        "roofline": roofline,
        "ms_per_step_steady": round(steady, 4) if steady is not None else None,
        "ms_per_step_amortised": round(ms_amortised, 4) if ms_amortised is not None else None,
        "value_amortised": round(I / (ms_amortised * 1e-3) / 1e9, 4) if ms_amortised is not None else None,
        "ms_per_step_with_kernel_events": round(ms_per_step_profiled, 4),
        "refresh_ms": round(refresh_ms, 4),
        "copy_kernel_GBps": round(copy_gbs, 1),
        "tile_stream_GBps": round(tile_gbs, 1) if tile_gbs is not None else None,
        "mfma_loop_TFLOPs": {k: round(v, 1) for k, v in mfma_tf.items()},
        "select": select_summary,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
