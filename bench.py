#!/usr/bin/env python3
"""bench.py -- one-GPU throughput of the verifiable-training hot path on MI355X.

Headline workload (the configuration the metric is quoted on): the GPT-2 117M MLP up-projection of one
training step, X 8192x768 ~ N(0,1) times W 768x3072 ~ N(0, 0.02^2) (+ zero bias), FP64.
One "step" is one pass of the whole path over that batch:
    trainer : vt_gemm_f64_round_log (variant 0, per-layer tau)  -> FP32 outputs + decision log
    auditor : vt_gemm_f64_round_log (variant 1: other accumulation order) -> its own FP64 results
              vt_round_replay of the trainer's log on them        -> FP32 outputs (must match)
    offline parts of the method run on the same tensors each step so every kernel is exercised:
              vt_threshold_stats(trainer FP64, auditor FP64), vt_round_log (standalone) on the
              auditor's FP64 results.
`value` is the metric as named: 2 M N K over the time of the fused trainer call (the GEMM with its
round/log epilogue plus the kernels that turn its decision bits into the ordered log), measured with
HIP events on the launch stream inside the timed steps.  The whole five-call step is reported beside it.
Other legs: the same call at fixed thresholds (tau_sweep), config 1 as latencies, config 5 (2^28 values,
thr 1 and 32) with the streaming ceiling, config 3 (GPT-2 layer stream with a per-op, per-layer adaptive
threshold), the linear layers' backward GEMMs, config 4 (ResNet-50 convolutions, per-layer roofline), and
the CPU oracle on the host's cores.  Inputs are resident in HBM before every timed region.  ONE JSON line.
"""
from __future__ import annotations

import argparse
import ctypes as C
import json
import multiprocessing as mp
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP64_MFMA_PEAK_TFLOPS = 78.6      # MI355X published dense FP64 matrix peak
HBM_PEAK_GBS = 8000.0             # MI355X published HBM3E bandwidth
TRAFFIC_PROFILE = "profiles/gemm_round_planes_gpt2_mlp_up_counters.md"


class HipEvents:
    """Raw hipEvent_t handles through the HIP runtime the library itself is linked to."""

    def __init__(self, lib):
        self.lib = lib
        lib.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        lib.hipEventRecord.argtypes = [C.c_void_p, C.c_void_p]
        lib.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        lib.hipEventSynchronize.argtypes = [C.c_void_p]

    def create(self):
        e = C.c_void_p()
        assert self.lib.hipEventCreate(C.byref(e)) == 0
        return e.value

    def record(self, e, stream):
        assert self.lib.hipEventRecord(C.c_void_p(e), C.c_void_p(stream)) == 0

    def elapsed_ms(self, a, b):
        assert self.lib.hipEventSynchronize(C.c_void_p(b)) == 0
        ms = C.c_float()
        assert self.lib.hipEventElapsedTime(C.byref(ms), C.c_void_p(a), C.c_void_p(b)) == 0
        return float(ms.value)


def committed_traffic():
    """HBM-side bytes per trainer-GEMM launch from the committed rocprofv3 counter summary
    (FETCH_SIZE and WRITE_SIZE passes of this same command, scaled against a plain copy), or None."""
    try:
        with open(os.path.join(ROOT, TRAFFIC_PROFILE)) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return int(line.split()[1])
    except (OSError, ValueError, IndexError):
        pass
    return None


def thr_layer_from(stats_u64) -> tuple[int, int, int, int]:
    """(thr_layer, n_flip, thr_flip, max_ulp64_diff) from the 68 integers of vt_threshold_stats: the library's
    rule (vt_thr_layer_from_stats), the smallest power-of-two threshold, capped at 1/4 ulp, that covers every
    observed divergence of the pair."""
    from paper_2403_09603_amd import vt_thr_layer_from_stats
    n_flip, thr_flip, max_diff = int(stats_u64[0]), int(stats_u64[1]), int(stats_u64[2])
    return vt_thr_layer_from_stats(thr_flip, max_diff), n_flip, thr_flip, max_diff


def resnet50_conv_layers():
    """The 53 convolutions of ResNet-50 at 224 x 224 (stride on the 3 x 3 of a stage's first block):
    (kind, input height = width, Cin, filter size, Cout, stride, padding)."""
    layers = [("7x7 first", 224, 3, 7, 64, 2, 3)]
    h, cin = 56, 64
    for width, blocks, stride in ((64, 3, 1), (128, 4, 2), (256, 6, 2), (512, 3, 2)):
        for b in range(blocks):
            s = stride if b == 0 else 1
            layers.append(("1x1", h, cin, 1, width, 1, 0))
            layers.append(("3x3", h, width, 3, width, s, 1))
            layers.append(("1x1", h // s, width, 1, 4 * width, 1, 0))
            if b == 0:
                layers.append(("1x1 downsample", h, cin, 1, 4 * width, s, 0))
            cin, h = 4 * width, h // s
    assert len(layers) == 53
    return layers


# ------------------------------------------------------------------------------------------------
# CPU oracle baseline.  The worker pool is forked before anything touches the GPU (a process that has
# initialised the GPU must not start others); the oracle itself is untouched: every worker runs the
# plain single-thread step on its own block of rows.
# ------------------------------------------------------------------------------------------------
_CPU = {}


def _cpu_init():
    import synth_inputs as si
    from oracle import vt_oracle as vo
    vo.lib()
    _CPU["X"], _CPU["W"], _CPU["bias"] = si.gpt2_mlp_up(config=2, rows=8192)


def _cpu_step_rows(job):
    """The benchmark step by the oracle on rows [lo, hi) of X: trainer GEMM + round/log, auditor GEMM
    (descending k) + replay, statistics of the pair, standalone round/log.  Returns replay mismatches."""
    from oracle import vt_oracle as vo
    lo, hi, tau = job
    if not _CPU:
        _cpu_init()
    Xs, W, bias = _CPU["X"][lo:hi], _CPU["W"], _CPU["bias"]
    cT = vo.gemm_f64(Xs, W, bias=bias, order=0)
    yT, idx, dirw, cnt = vo.round_log(cT, tau)
    cA = vo.gemm_f64(Xs, W, bias=bias, order=1)
    yA = vo.round_replay(cA, idx, dirw)
    vo.threshold_stats(cT, cA)
    vo.round_log(cA, tau)
    return int((yA.view(np.uint32) != yT.view(np.uint32)).sum())


def cpu_pool():
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    workers = max(1, min(16, cores))        # the GPU machine's CPU share for one GPU is 16
    pool = mp.get_context("fork").Pool(workers, initializer=_cpu_init)
    pool.map(_cpu_step_rows, [(0, 1, 0.25)] * workers)          # every worker up, inputs drawn, library loaded
    return pool, workers


def cpu_baseline(pool, workers, tau, M, N, K, rows_single):
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    if not _CPU:
        _cpu_init()
    t0 = time.perf_counter()
    mism1 = _cpu_step_rows((0, rows_single, tau))
    dt1 = time.perf_counter() - t0
    # all workers: one block of 2 * `rows_single` rows each (bounded sample: at most the whole batch)
    M = min(M, workers * 2 * rows_single)
    edges = [M * i // workers for i in range(workers + 1)]
    t0 = time.perf_counter()
    mism = sum(pool.map(_cpu_step_rows, [(edges[i], edges[i + 1], tau) for i in range(workers)], chunksize=1))
    dtn = time.perf_counter() - t0
    pool.close()
    pool.join()
    fl = 2 * 2.0 * N * K          # two GEMMs per row of X
    return {
        "value": round(fl * M / dtn / 1e12, 6), "unit": "TFLOP/s", "cores": workers, "kind": "oracle",
        "sample": f"the whole step (both GEMMs, round/log, replay, stats, standalone round/log) on the first {M} of 8192 rows of X, "
                  f"rows split over {workers} worker processes, each the plain single-thread oracle (oracle/vt_oracle.c): "
                  f"{dtn:.1f} s",
        "seconds": round(dtn, 2), "replay_mismatches": mism,
        "single_thread": {"value": round(fl * rows_single / dt1 / 1e12, 6), "unit": "TFLOP/s", "cores": 1,
                          "sample": f"the same step on the first {rows_single} rows: {dt1:.1f} s",
                          "seconds": round(dt1, 2), "replay_mismatches": mism1},
        "host": {"cpu_model": model, "logical_cpus": os.cpu_count(),
                 "cpus_in_affinity_mask": len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else None,
                 "workers_used": workers},
    }


# ------------------------------------------------------------------------------------------------
class Bench:
    def __init__(self, vt, torch, ev):
        self.vt, self.torch, self.ev = vt, torch, ev
        self.dev = "cuda:0"
        self.stats = torch.zeros(68, dtype=torch.int64, device=self.dev)

    def stream(self):
        return self.torch.cuda.current_stream().cuda_stream

    def per_call(self, fn, warm=5, reps=20, kernel_events=False):
        """Median and minimum time of one call (HIP events on the launch stream around each call),
        optionally with the call's main kernel alone (events recorded by the library itself)."""
        vt, ev, torch = self.vt, self.ev, self.torch
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        pairs = [(ev.create(), ev.create()) for _ in range(reps)]
        kpairs = [(ev.create(), ev.create()) for _ in range(reps)] if kernel_events else None
        s = self.stream()
        for i in range(reps):
            if kernel_events:
                vt.vt_set_kernel_events(*kpairs[i])
            ev.record(pairs[i][0], s)
            fn()
            ev.record(pairs[i][1], s)
            if kernel_events:
                vt.vt_set_kernel_events(None, None)
        torch.cuda.synchronize()
        call = [ev.elapsed_ms(a, b) for a, b in pairs]
        out = {"median_ms": float(np.median(call)), "min_ms": float(np.min(call))}
        if kernel_events:
            out["kernel_median_ms"] = float(np.median([ev.elapsed_ms(a, b) for a, b in kpairs]))
        return out

    def read_stats(self):
        self.torch.cuda.synchronize()
        return self.stats.cpu().numpy().view(np.uint64)

    def up(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)


def r4(v):
    return round(float(v), 4)


# ------------------------------------------------------------------------------------------------
def leg_config2(b: Bench, args, si):
    """Config 2 (headline).  Returns (json fields, tau, keep-alive tensors for the sweep)."""
    vt, torch, ev = b.vt, b.torch, b.ev
    M, K, N = 8192, 768, 3072
    seeds = {"X": si.seed_for(2, 0), "W": si.seed_for(2, 1)}
    X, W, bias = si.gpt2_mlp_up(config=2, rows=M)
    Xd, Wd, bd = b.up(X), b.up(W), b.up(bias)
    dev = b.dev
    C32_T = torch.empty((M, N), dtype=torch.float32, device=dev)
    C32_A = torch.empty((M, N), dtype=torch.float32, device=dev)
    y_A = torch.empty(M * N, dtype=torch.float32, device=dev)
    y_S = torch.empty(M * N, dtype=torch.float32, device=dev)
    C64_T = torch.empty((M, N), dtype=torch.float64, device=dev)
    C64_A = torch.empty((M, N), dtype=torch.float64, device=dev)
    total = M * N
    log_T, log_A, log_S = vt.alloc_log(total), vt.alloc_log(0), vt.alloc_log(total)
    ws_g = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, 1))
    ws_r = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, total))

    def gemm(variant, tau, c32, c64, log):
        vt.vt_gemm_f64_round_log(False, False, M, N, K, 1.0, Xd, K, 0, Wd, N, 0, bd, 1, c32, N, 0, c64,
                                 variant, tau, log, ws_g)

    # per-layer threshold (untimed set-up): statistics of the trainer/auditor pair, then the
    # smallest power-of-two threshold that covers every observed divergence
    gemm(0, 0.0, C32_T, C64_T, log_A)
    gemm(1, 0.0, C32_A, C64_A, log_A)
    vt.vt_threshold_stats(C64_T, C64_A, b.stats)
    thr, n_flip, thr_flip, max_diff = thr_layer_from(b.read_stats())
    tau = thr * 2.0 ** -29
    gemm(0, tau, C32_T, None, log_T)
    torch.cuda.synchronize()
    count_T = log_T.read_count()

    def step(i=None):
        s = b.stream()
        if i is not None:
            vt.vt_set_kernel_events(*kern[i])
            ev.record(call[i][0], s)
        gemm(0, tau, C32_T, None, log_T)                               # trainer: a1 + a2 + a3
        if i is not None:
            ev.record(call[i][1], s)
            vt.vt_set_kernel_events(None, None)
        gemm(1, 0.0, C32_A, C64_A, log_A)                               # auditor's own layer
        vt.vt_round_replay(C64_A.view(-1), log_T.idx, log_T.dir, count_T, y_A)   # a5
        vt.vt_threshold_stats(C64_T.view(-1), C64_A.view(-1), b.stats)  # a6
        vt.vt_round_log(C64_A.view(-1), tau, y_S, log_S, ws_r)          # a4

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    call = [(ev.create(), ev.create()) for _ in range(args.steps)]
    kern = [(ev.create(), ev.create()) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    call_ms = [ev.elapsed_ms(a, c) for a, c in call]
    kern_ms = [ev.elapsed_ms(a, c) for a, c in kern]
    call_mean, gemm_mean = float(np.mean(call_ms)), float(np.mean(kern_ms))

    # correctness of what was timed (untimed): the auditor ends bit-identical to the trainer
    mism = int((y_A.view(torch.int32) != C32_T.view(-1).view(torch.int32)).sum().item())
    count_S = log_S.read_count()
    flops = 2.0 * M * N * K
    value = flops / (call_mean * 1e-3) / 1e12
    achieved = flops / (gemm_mean * 1e-3) / 1e12
    out = {
        "metric": "fused FP64 GEMM+round+log TFLOP/s",
        "value": round(value, 3), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r4(ms_per_step), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "value_definition": "2 M N K / mean time of the fused trainer call inside the timed steps (HIP events on the launch "
                            "stream around vt_gemm_f64_round_log: gemm_round_planes_kernel + seg_count + seg_scan + compact)",
        "config": {"workload": "config 2: GPT-2 117M MLP up-projection, X 8192x768 @ W 768x3072 (+bias), FP64 -> FP32 round + "
                               "sparse decision log at the per-layer threshold",
                   "M": M, "N": N, "K": K, "seeds": seeds, "tau_ulp": tau, "thr": thr, "logged": count_T,
                   "logged_fraction": round(count_T / total, 6), "n_flip": n_flip, "thr_flip": thr_flip,
                   "max_ulp64_diff": max_diff, "replay_mismatches": mism,
                   "log_bytes": count_T * 4 + (count_T + 7) // 8,
                   "trainer_call_ms": r4(call_mean), "trainer_call_ms_median": r4(np.median(call_ms)),
                   "trainer_call_frac_mfma_peak": r4(value / FP64_MFMA_PEAK_TFLOPS),
                   "step_calls": "trainer fused GEMM; auditor GEMM (variant 1, FP64 out); replay of the trainer's log; "
                                 "threshold statistics of the pair; standalone round/log of the auditor's FP64 tensor",
                   "step_ms": r4(ms_per_step),
                   "step_TFLOPs_two_gemms": round(2 * flops / (ms_per_step * 1e-3) / 1e12, 3),
                   "step_standalone_log_entries": count_S},
        "roofline": {"bound": "mfma", "kernel": "gemm_round_planes_kernel (trainer, variant 0), the dominant kernel of the call",
                     "achieved": round(achieved, 3), "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": r4(achieved / FP64_MFMA_PEAK_TFLOPS), "kernel_ms": r4(gemm_mean),
                     "call": {"kernels": "gemm_round_planes_kernel + compact_onepass_kernel",
                              "ms": r4(call_mean), "achieved": round(value, 3), "frac": r4(value / FP64_MFMA_PEAK_TFLOPS)},
                     "algorithmic_bytes": 8 * (M * K + K * N + N) + 4 * M * N + 2 * (M * ((N + 63) // 64) * 8),
                     "traffic": committed_traffic(),
                     "traffic_source": TRAFFIC_PROFILE + " (rocprofv3 FETCH_SIZE/WRITE_SIZE of this command; not measured in this run)"},
    }

    # ---- the same trainer call at three fixed thresholds (sparse, medium and the paper's default band),
    # both log formats: call time and log size
    sweep = []
    dlog_T = vt.alloc_dense_log(total)
    for name, tau_b in (("2^-24", 2.0 ** -24), ("2^-8", 2.0 ** -8), ("1/4", 0.25)):
        row = {"tau_ulp": name, "thr": vt.vt_thr_from_tau(tau_b)}
        for fmt, lg in (("sparse", log_T), ("packed", dlog_T)):
            t = b.per_call(lambda: gemm(0, tau_b, C32_T, None, lg), warm=40, reps=20)
            cnt_b = lg.read_count()
            row["logged"] = cnt_b
            row[fmt + "_call_ms"] = r4(t["median_ms"])
            row[fmt + "_call_ms_min"] = r4(t["min_ms"])
            row[fmt + "_log_bytes"] = cnt_b * 4 + (cnt_b + 7) // 8 if fmt == "sparse" else (total + 4) // 5
        sweep.append(row)
    out["tau_sweep"] = {"timing": "40 warm-up + 20 timed calls each, HIP events around every call: median and minimum",
                        "rows": sweep}
    return out, tau, (X, W, bias)


def leg_config1(b: Bench, si):
    """Config 1 as latencies: 256^3 fused GEMM, a 2^20-value vector through round/log and replay."""
    vt, torch = b.vt, b.torch
    dev = b.dev
    A, B = si.tiny_gemm()
    Ad, Bd = b.up(A), b.up(B)
    M = N = K = 256
    c32 = torch.empty((M, N), dtype=torch.float32, device=dev)
    c64 = [torch.empty((M, N), dtype=torch.float64, device=dev) for _ in range(2)]
    log = vt.alloc_log(M * N)
    ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, 1))

    def gemm(variant, tau, c, lg):
        vt.vt_gemm_f64_round_log(False, False, M, N, K, 1.0, Ad, K, 0, Bd, N, 0, None, 1, c32, N, 0, c, variant, tau, lg, ws)
    gemm(0, 0.0, c64[0], log)
    gemm(1, 0.0, c64[1], log)
    vt.vt_threshold_stats(c64[0], c64[1], b.stats)
    thr, n_flip, thr_flip, max_diff = thr_layer_from(b.read_stats())
    tau = thr * 2.0 ** -29
    tg = b.per_call(lambda: gemm(0, tau, None, log), warm=10, reps=50)
    cnt_g = log.read_count()
    # host-inclusive: call + synchronise, wall clock
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(50):
        gemm(0, tau, None, log)
        torch.cuda.synchronize()
    wall_us = (time.perf_counter() - t0) / 50 * 1e6
    n = 1 << 20
    x = si.normal(n, si.seed_for(1, 2))
    xd = b.up(x)
    y = torch.empty(n, dtype=torch.float32, device=dev)
    vlog = vt.alloc_log(n)
    wsr = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    rows = {}
    for name, tau_v in (("tau_2^-30", 2.0 ** -30), ("tau_2^-4", 2.0 ** -4)):
        t = b.per_call(lambda: vt.vt_round_log(xd, tau_v, y, vlog, wsr), warm=10, reps=50)
        cnt = vlog.read_count()
        tr = b.per_call(lambda: vt.vt_round_replay(xd, vlog.idx, vlog.dir, cnt, y), warm=10, reps=50)
        rows[name] = {"thr": vt.vt_thr_from_tau(tau_v), "logged": cnt, "round_log_us": round(t["median_ms"] * 1e3, 2),
                      "round_log_us_min": round(t["min_ms"] * 1e3, 2), "replay_us": round(tr["median_ms"] * 1e3, 2)}
    return {"workload": "config 1: A, B 256x256 ~ N(0,1); vector of 2^20 ~ N(0,1) (cache-resident: latencies, not bandwidth)",
            "seeds": {"A": si.seed_for(1, 0), "B": si.seed_for(1, 1), "x": si.seed_for(1, 2)},
            "gemm_256": {"thr_layer": thr, "n_flip": n_flip, "thr_flip": thr_flip, "max_ulp64_diff": max_diff, "logged": cnt_g,
                         "fused_call_us": round(tg["median_ms"] * 1e3, 2), "fused_call_us_min": round(tg["min_ms"] * 1e3, 2),
                         "call_and_synchronise_wall_us": round(wall_us, 1)},
            "vector_2p20": rows,
            "note": "tau = 2^-30 ulp is below FP64 resolution: thr = 1, exact ties only, so the log of a random vector is empty"}


def leg_config5(b: Bench, si, hashes=True):
    """Config 5: 2^28 values, a tenth planted inside the band, for thr = 1 (tau_ulp = 2^-40 and 2^-32 both quantise to it)
    and thr = 32 (2^-24); the streaming ceiling; packed log, fused layers, b_r = 26 and the checkpoint hash at thr = 32."""
    vt, torch = b.vt, b.torch
    dev = b.dev
    n = 1 << 28
    y1 = torch.empty(n, dtype=torch.float32, device=dev)
    y2 = torch.empty(n, dtype=torch.float32, device=dev)
    logs = vt.alloc_log(n // 4)
    wss = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
    res = {"workload": "config 5: 2^28 FP64 values, 10% planted within thr FP64 steps of an FP32 midpoint (2^-10 more just outside), "
                       "rest N(0,1); the auditor's copy moved by a seeded integer in (-thr, thr) steps",
           "n": n, "seeds": {"x": si.seed_for(5, 0), "perturbation": si.seed_for(5, 1)},
           "timing": "10 warm-up + 20 timed calls, HIP events around every call, median"}
    ceiling = None
    by_thr = {}
    keep = None
    for thr_s, taus in ((1, "2^-40 and 2^-32 ulp (both below FP64 resolution: exact ties only)"), (32, "2^-24 ulp")):
        x, _ = si.planted_vector(n, si.seed_for(5, 0), thr=thr_s)
        xa = si.perturb_steps(x, si.seed_for(5, 1), thr_s)
        xd, xad = b.up(x), b.up(xa)
        del x, xa
        tau_s = thr_s * 2.0 ** -29
        if ceiling is None:
            # the practical ceiling: the library's round-only stream (tau = 0 logs nothing, so vt_round_log runs a plain
            # FP64 -> FP32 convert-copy in the launch shape that measured fastest on this part: 8 B in, 4 B out)
            empty = vt.alloc_log(0)
            tc = b.per_call(lambda: vt.vt_round_log(xd, 0.0, y1, empty, wss), warm=10, reps=20, kernel_events=True)
            ceiling = n * 12 / tc["kernel_median_ms"] * 1e-6
            res["ceiling_convert_copy"] = {"what": "vt_round_log with tau = 0 (round only, the fastest plain convert-copy shape found: 8 B read + 4 B written per value)",
                                           "kernel_ms": r4(tc["kernel_median_ms"]), "call_ms": r4(tc["median_ms"]),
                                           "GBs": round(ceiling, 1), "frac_hbm": r4(ceiling / HBM_PEAK_GBS)}
        rl = b.per_call(lambda: vt.vt_round_log(xd, tau_s, y1, logs, wss), warm=10, reps=20, kernel_events=True)
        cnt = logs.read_count()
        rp = b.per_call(lambda: vt.vt_round_replay(xad, logs.idx, logs.dir, cnt, y2), warm=10, reps=20, kernel_events=True)
        mism = int((y1.view(torch.int32) != y2.view(torch.int32)).sum().item())
        st = b.per_call(lambda: vt.vt_threshold_stats(xd, xad, b.stats), warm=10, reps=20)
        s = b.read_stats()
        rho = cnt / n
        bytes_rl = n * (8 + 4 + rho * 4.125)

        def rate(ms, nbytes=bytes_rl):
            g = nbytes / ms * 1e-6
            return {"ms": r4(ms), "GBs": round(g, 1), "frac_hbm": r4(g / HBM_PEAK_GBS), "frac_ceiling": r4(g / ceiling)}
        by_thr[f"thr_{thr_s}"] = {
            "tau_ulp": taus, "logged_fraction": round(rho, 6), "log_bytes_per_element": round(rho * 4.125, 4),
            "round_log": {**rate(rl["median_ms"]), "main_kernel": rate(rl["kernel_median_ms"])},
            "replay": {**rate(rp["median_ms"]), "main_kernel": rate(rp["kernel_median_ms"])},
            "stats": rate(st["median_ms"], n * 16),
            "replay_mismatches": mism, "pair_n_flip": int(s[0]), "pair_thr_flip": int(s[1]), "pair_max_ulp64_diff": int(s[2])}
        if thr_s == 32:
            keep = (xd, xad, tau_s)
        else:
            del xd, xad
    res["sparse_log"] = by_thr
    xd, xad, tau_s = keep

    def timed(fn, reps=20):
        t = b.per_call(fn, warm=10, reps=reps)
        return t["median_ms"]

    # the same tensor (thr = 32) with the log in the paper's packed ternary form (five entries per byte)
    dlog = vt.alloc_dense_log(n)
    rd = timed(lambda: vt.vt_round_log(xd, tau_s, y1, dlog, wss))
    pd = timed(lambda: vt.vt_round_replay_dense(xad, dlog.dense, y2))
    mism_d = int((y1.view(torch.int32) != y2.view(torch.int32)).sum().item())
    cnt_d = dlog.read_count()
    bytes_d = n * (8 + 4 + 0.2)
    res["packed_ternary_log"] = {
        "thr": 32, "log_bytes_per_element": 0.2, "logged": cnt_d,
        "round_log_ms": r4(rd), "round_log_GBs": round(bytes_d / rd * 1e-6, 1), "round_log_frac_hbm": r4(bytes_d / rd * 1e-6 / HBM_PEAK_GBS),
        "round_log_frac_ceiling": r4(bytes_d / rd * 1e-6 / ceiling),
        "replay_ms": r4(pd), "replay_GBs": round(bytes_d / pd * 1e-6, 1), "replay_frac_hbm": r4(bytes_d / pd * 1e-6 / HBM_PEAK_GBS),
        "replay_frac_ceiling": r4(bytes_d / pd * 1e-6 / ceiling), "replay_mismatches": mism_d}
    # rounding amount b_r = 26 (six more mantissa bits dropped), packed log
    dlog26 = vt.alloc_dense_log(n)
    dlog26.b_r = 26
    r26 = timed(lambda: vt.vt_round_log(xd, tau_s, y1, dlog26, wss), reps=5)
    p26 = timed(lambda: vt.vt_round_replay_dense(xd, dlog26.dense, y2, b_r=26), reps=5)
    mism_26 = int((y1.view(torch.int32) != y2.view(torch.int32)).sum().item())
    s26 = timed(lambda: vt.vt_threshold_stats(xd, xad, b.stats, b_r=26), reps=5)
    res["b_r_26_packed_log"] = {
        "round_log_ms": r4(r26), "round_log_GBs": round(bytes_d / r26 * 1e-6, 1),
        "replay_ms": r4(p26), "replay_GBs": round(bytes_d / p26 * 1e-6, 1),
        "stats_ms": r4(s26), "stats_GBs": round(n * 16 / s26 * 1e-6, 1), "replay_mismatches": mism_26}
    del dlog26
    # fused layers (FP64 evaluation + hook in one pass, packed log) over the same 2^28 values seen as 262144 rows of 1024
    rows_l, cols_l = n // 1024, 1024
    wsl = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, rows_l, cols_l))
    wsb = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, n // 64, 64))
    layers = {}
    for lname, lop, shape, reads, kw in (
            ("gelu_tanh", vt.VT_LAYER_GELU_TANH, (rows_l, cols_l), 1, {}),
            ("layer_norm", vt.VT_LAYER_NORM, (rows_l, cols_l), 1, {"eps": 1e-5}),
            ("softmax", vt.VT_LAYER_SOFTMAX, (rows_l, cols_l), 1, {"scale": 0.125}),
            ("batch_norm_relu_64ch", vt.VT_LAYER_BATCHNORM_RELU, (n // 64, 64), 2, {"eps": 1e-5})):
        wsx = wsb if shape[1] == 64 else wsl
        lt = timed(lambda: vt.vt_layer_f64_round_log(lop, xd, None, None, None, shape[0], shape[1], y1, None, 0,
                                                     tau_s, dlog, wsx, **kw), reps=5)
        # reads of the input from memory: batch norm takes its column statistics in a pass of its own before the
        # fused pass; layer norm and softmax over rows this short are computed a row at a time from registers
        lbytes = n * (8 * reads + 4 + 0.2)
        layers[lname] = {"ms": r4(lt), "input_reads": reads, "GBs": round(lbytes / lt * 1e-6, 1),
                         "frac_hbm": r4(lbytes / lt * 1e-6 / HBM_PEAK_GBS)}
    res["fused_layers_packed_log"] = layers
    del wsl, wsb
    if hashes:
        # checkpoint hash: SHA-256 chunk tree over as many bytes as GPT-2 117M has FP32 weights (the first bytes of
        # the resident vector), then the Merkle root over 1024 checkpoint leaves
        hbytes = 124_439_808 * 4
        hsrc = xd.view(torch.uint8)[:hbytes]
        digest = torch.zeros(32, dtype=torch.uint8, device=dev)
        hs = {"bytes": hbytes}
        for chunk in (1024, 4096):
            wsh = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_SHA256_TREE, 1, hbytes, chunk))
            ht = timed(lambda: vt.vt_sha256_tree(hsrc, chunk, digest, wsh), reps=5)
            hs[f"sha256_tree_chunk{chunk}"] = {"ms": r4(ht), "GBs": round(hbytes / ht * 1e-6, 1)}
        leaves = xd.view(torch.uint8)[:1024 * 32]
        wsm = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_MERKLE_ROOT, 1, 1024))
        hs["merkle_root_1024_leaves_ms"] = r4(timed(lambda: vt.vt_merkle_root(leaves, digest, wsm), reps=5))
        res["checkpoint_hash"] = hs
    return res


# ------------------------------------------------------------------------------------------------
def run_stream(b: Bench, calls, reps=4, graph=True):
    """calls: list of (kind, flops, fn).  Runs the stream `reps` times, times the last pass as a whole and per
    call (events on the stream the library launches on), then the same stream replayed from a HIP graph."""
    torch = b.torch
    for _ in range(reps - 1):
        for _, _, fn in calls:
            fn()
    torch.cuda.synchronize()
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
    evs[0].record()
    for i, (_, _, fn) in enumerate(calls):
        fn()
        evs[i + 1].record()
    torch.cuda.synchronize()
    total_ms = evs[0].elapsed_time(evs[-1])
    per_call = [evs[i].elapsed_time(evs[i + 1]) for i in range(len(calls))]
    kinds = {}
    for (kind, fl, _), ms in zip(calls, per_call):
        k = kinds.setdefault(kind, [0, 0.0, 0.0])
        k[0] += 1; k[1] += fl; k[2] += ms
    flops = sum(fl for _, fl, _ in calls)
    res = {"calls": len(calls), "TFLOP": round(flops / 1e12, 4), "ms": round(total_ms, 3),
           "TFLOPs": round(flops / total_ms / 1e9, 2),
           "frac_mfma_peak": r4(flops / total_ms / 1e9 / FP64_MFMA_PEAK_TFLOPS),
           "by_kind": {k: {"calls": v[0], "ms": round(v[2], 3), "TFLOPs": round(v[1] / v[2] / 1e9, 2),
                           "frac_mfma_peak": r4(v[1] / v[2] / 1e9 / FP64_MFMA_PEAK_TFLOPS)} for k, v in kinds.items()}}
    if graph:
        # the library allocates nothing and never synchronises, so its calls can be captured: what launch gaps cost
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _, _, fn in calls:
                fn()
        g.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record(); g.replay(); g1.record()
        torch.cuda.synchronize()
        gms = g0.elapsed_time(g1)
        del g
        res["graph_replay_ms"] = round(gms, 3)
        res["graph_replay_TFLOPs"] = round(flops / gms / 1e9, 2)
    return res, per_call


def leg_gpt2(b: Bench, si):
    """Config 3: the GPT-2 117M layer stream, 12 layers x (QKV, scores, attention output, MLP up, MLP down), every call
    at a threshold chosen for that op of that layer from vt_threshold_stats over its two accumulation orders.
    Then the backward GEMMs of the linear layers (tau = 1/4, packed log)."""
    vt, torch = b.vt, b.torch
    dev = b.dev
    T, D, H, DH, B = 1024, 768, 12, 64, 8
    R = B * T
    big = max(R * 4 * D, B * H * T * T)
    c32 = torch.empty(big, dtype=torch.float32, device=dev)
    c64 = [torch.empty(big, dtype=torch.float64, device=dev) for _ in range(2)]
    slog = vt.alloc_log(big)
    dlog = vt.alloc_dense_log(big)
    none = vt.alloc_log(0)
    ws = vt.alloc_workspace(max(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, R, 4 * D, D, 1),
                                vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, R, D, 4 * D, 1),
                                vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, T, T, DH, B * H)))
    f32grid = lambda a: a.astype(np.float32).astype(np.float64)
    shapes = {"qkv": (D, 3 * D), "attn_out": (D, D), "mlp_up": (D, 4 * D), "mlp_down": (4 * D, D)}
    calls, table, seeds = [], [], []
    log_sparse = log_packed = log_chosen = 0
    outputs = 0
    keep = []
    for layer in range(12):
        base = 64 * layer                          # tensor ordinals of this layer (config 3)
        seeds.append(si.seed_for(3, base))
        act = b.up(f32grid(si.normal((R, D), si.seed_for(3, base + 0))))
        act4 = b.up(f32grid(si.normal((R, 4 * D), si.seed_for(3, base + 1))))
        qkv = b.up(f32grid(si.normal((R, 3 * D), si.seed_for(3, base + 2)))).view(-1)    # a rounded QKV output
        wts = {nm: b.up(si.normal(s, si.seed_for(3, base + 3 + i), 0.02)) for i, (nm, s) in enumerate(shapes.items())}
        bias = {nm: torch.zeros(s[1], dtype=torch.float64, device=dev) for nm, s in shapes.items()}
        keep.append((act, act4, qkv, wts, bias))

        def linear(nm, x):
            w = wts[nm]
            k, n = w.shape
            bs = bias[nm]
            return (nm, 2.0 * R * n * k, R * n,
                    lambda variant, tau, c, lg: vt.vt_gemm_f64_round_log(False, False, R, n, k, 1.0, x, k, 0, w, n, 0, bs, 1,
                                                                         c32, n, 0, c, variant, tau, lg, ws))

        def scores(qkv):
            # Q and K of (sequence, head) are column slices of the QKV activation: heads 64 columns apart,
            # sequences T rows apart -- one nested-batch call covers all 96 matrices
            return ("scores", 2.0 * B * H * T * T * DH, B * H * T * T,
                    lambda variant, tau, c, lg: vt.vt_gemm_f64_round_log_nested(
                        False, True, T, T, DH, 0.125, qkv, 3 * D, DH, T * 3 * D, qkv[D:], 3 * D, DH, T * 3 * D, None, H, B,
                        c32, T, T * T, c, variant, tau, lg, ws))

        for nm, fl, nout, fn in (linear("qkv", act), scores(qkv), linear("attn_out", act), linear("mlp_up", act),
                                 linear("mlp_down", act4)):
            # Algorithm "threshold", collection loop: the op on two "devices" (accumulation orders), statistics of the pair
            fn(0, 0.0, c64[0], none)
            fn(1, 0.0, c64[1], none)
            vt.vt_threshold_stats(c64[0][:nout], c64[1][:nout], b.stats)
            thr, n_flip, thr_flip, max_diff = thr_layer_from(b.read_stats())
            tau = thr * 2.0 ** -29
            fn(0, tau, None, dlog)
            torch.cuda.synchronize()
            cnt = dlog.read_count()
            sp, pk = cnt * 4 + (cnt + 7) // 8, (nout + 4) // 5
            lg = slog if sp < pk else dlog          # the smaller of the two log formats for this op
            log_sparse += sp; log_packed += pk; log_chosen += min(sp, pk); outputs += nout
            calls.append((nm, fl, lambda fn=fn, tau=tau, lg=lg: fn(0, tau, None, lg)))
            table.append({"layer": layer, "op": nm, "thr_layer": thr, "thr_flip": thr_flip, "n_flip": n_flip,
                          "max_ulp64_diff": max_diff, "logged_fraction": round(cnt / nout, 5),
                          "log": "sparse" if sp < pk else "packed"})
    res, per_call = run_stream(b, calls)
    for row, ms in zip(table, per_call):
        row["ms"] = r4(ms)
    # per op type: the thresholds chosen over the 12 layers
    by_op = {}
    for row in table:
        o = by_op.setdefault(row["op"], {"thr_layer": [], "thr_flip": [], "logged_fraction": []})
        for k in o:
            o[k].append(row[k])
    res["adaptive_threshold"] = {
        "rule": "per op and layer: vt_threshold_stats over variants 0 and 1, thr_layer = vt_thr_layer_from_stats = min(2^27, next_pow2(max(thr_flip, "
                "max_ulp64_diff + 1))) (guarantees replay on the observed pair); thr_flip is the paper's rule (flips only)",
        "by_op": {k: {"thr_layer_min": min(v["thr_layer"]), "thr_layer_max": max(v["thr_layer"]),
                      "thr_flip_max": max(v["thr_flip"]),
                      "logged_fraction_mean": round(float(np.mean(v["logged_fraction"])), 5)} for k, v in by_op.items()},
        "per_call": table}
    res["log_bytes"] = {"fp32_output_bytes": outputs * 4, "sparse_format_total": log_sparse, "packed_format_total": log_packed,
                        "smaller_per_op_total": log_chosen}
    res["workload"] = ("config 3: 12 layers x (QKV 768->2304, scores Q K^T / 8 per head as strided slices of a rounded QKV "
                       "activation, attention output 768->768, MLP 768->3072->768), batch 8 x 1024 tokens; own seeded operands per layer")
    res["seeds"] = {"layer_l_tensor_i": "0x240309603000 + 16*3 + 64*l + i  (i: act, act4, qkv, W_qkv, W_attn_out, W_mlp_up, W_mlp_down)",
                    "first_per_layer": seeds}
    out = {"gpt2_117m_layer_stream": res}

    # ---- backward GEMMs of the same linear layers (last layer's operands): dX = dY W^T (B transposed) and dW = X^T dY
    # (A transposed, K = 8192 tokens: deterministic split-K), each output rounded and logged like the forward ones
    act, act4, qkv, wts, bias = keep[-1]
    del keep
    gy = {nm: b.up(si.normal((R, w.shape[1]), si.seed_for(3, 800 + i), 1e-3)) for i, (nm, w) in enumerate(wts.items())}
    xin = {"qkv": act, "attn_out": act, "mlp_up": act, "mlp_down": act4}
    ws_b = vt.alloc_workspace(max(max(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, R, w.shape[0], w.shape[1], 1),
                                      vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, w.shape[0], w.shape[1], R, 1))
                                  for w in wts.values()))
    tau = 0.25

    def backward(nm):
        w = wts[nm]
        k, n = w.shape
        return [(nm + " dX", 2.0 * R * n * k,
                 lambda: vt.vt_gemm_f64_round_log(False, True, R, k, n, 1.0, gy[nm], n, 0, w, n, 0, None, 1, c32, k, 0,
                                                  None, 0, tau, dlog, ws_b)),
                (nm + " dW", 2.0 * R * n * k,
                 lambda: vt.vt_gemm_f64_round_log(True, False, k, n, R, 1.0, xin[nm], k, 0, gy[nm], n, 0, None, 1, c32, n, 0,
                                                  None, 0, tau, dlog, ws_b))]
    calls = []
    for _ in range(12):
        for nm in ("mlp_down", "mlp_up", "attn_out", "qkv"):
            calls += backward(nm)
    res_b, _ = run_stream(b, calls)
    res_b["workload"] = ("input and weight gradients of the four linear layers of each of 12 blocks, batch 8 x 1024 tokens, "
                         "tau = 1/4 ulp, packed log; grad-output seeds 0x240309603000 + 16*3 + 800 + i")
    out["gpt2_117m_linear_backward"] = res_b
    return out


def leg_gpt2_block(b: Bench, si):
    """One whole GPT-2 117M block forward at batch 8 x 1024 tokens, every intermediate rounded and logged (tau = 1/4 ulp,
    packed log): the five GEMMs of config 3 plus what stands between them -- layer norms, causal softmax, the
    probabilities-times-values product per head, GELU, residual additions.  Every op has seeded operands of its own on
    the FP32 grid (a real block would feed each op the FP32 output of the one before)."""
    vt, torch = b.vt, b.torch
    dev = b.dev
    T, D, H, DH, B = 1024, 768, 12, 64, 8
    R = B * T
    tau = 0.25
    f32grid = lambda a: a.astype(np.float32).astype(np.float64)
    seed = lambda i: si.seed_for(3, 900 + i)
    x = b.up(f32grid(si.normal((R, D), seed(0))))
    x2 = b.up(f32grid(si.normal((R, D), seed(1))))
    h4 = b.up(f32grid(si.normal((R, 4 * D), seed(2))))
    qkv = b.up(f32grid(si.normal((R, 3 * D), seed(3)))).view(-1)
    logits = b.up(f32grid(si.normal(B * H * T * T, seed(4), 2.0)))                      # pre-softmax scores, already scaled
    probs = b.up(f32grid(np.abs(si.normal(B * H * T * T, seed(5))) * (2.0 / T)))     # rows of about unit mass
    gamma = b.up(f32grid(1.0 + 0.1 * si.normal(D, seed(6))))
    beta = b.up(f32grid(0.1 * si.normal(D, seed(7))))
    shapes = {"qkv": (D, 3 * D), "attn_out": (D, D), "mlp_up": (D, 4 * D), "mlp_down": (4 * D, D)}
    wts = {nm: b.up(si.normal(sh, seed(8 + i), 0.02)) for i, (nm, sh) in enumerate(shapes.items())}
    bias = {nm: torch.zeros(sh[1], dtype=torch.float64, device=dev) for nm, sh in shapes.items()}
    big = B * H * T * T
    y32 = torch.empty(big, dtype=torch.float32, device=dev)
    dlog = vt.alloc_dense_log(big)
    ws = vt.alloc_workspace(max(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, R, 4 * D, D, 1),
                                vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, R, D, 4 * D, 1),
                                vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, T, T, DH, B * H),
                                vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, T, DH, T, B * H),
                                vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, B * H * T, T),
                                vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, R, 4 * D)))

    def linear(nm, a):
        w = wts[nm]
        k, n = w.shape
        return (nm, 2.0 * R * n * k, 8.0 * (R * k + k * n) + 4.2 * R * n,
                lambda: vt.vt_gemm_f64_round_log(False, False, R, n, k, 1.0, a, k, 0, w, n, 0, bias[nm], 1, y32, n, 0, None, 0,
                                                 tau, dlog, ws))

    def layer(nm, op, a, rows, cols, reads=1, second=None, **kw):
        g, be = (gamma, beta) if op == vt.VT_LAYER_NORM else (None, None)
        return (nm, 0.0, rows * cols * (8.0 * reads + 4.2),
                lambda: vt.vt_layer_f64_round_log(op, a, second, g, be, rows, cols, y32, None, 0, tau, dlog, ws, **kw))

    ops = [
        layer("layer_norm_1", vt.VT_LAYER_NORM, x, R, D, eps=1e-5),
        linear("qkv", x),
        ("scores", 2.0 * B * H * T * T * DH, 8.0 * 2 * R * D + 4.2 * B * H * T * T,
         lambda: vt.vt_gemm_f64_round_log_nested(False, True, T, T, DH, 0.125, qkv, 3 * D, DH, T * 3 * D, qkv[D:], 3 * D, DH,
                                                 T * 3 * D, None, H, B, y32, T, T * T, None, 0, tau, dlog, ws)),
        layer("softmax_causal", vt.VT_LAYER_SOFTMAX, logits, B * H * T, T, scale=1.0, causal_period=T),
        ("probs_times_values", 2.0 * B * H * T * T * DH, 8.0 * (B * H * T * T + R * D) + 4.2 * R * D,
         lambda: vt.vt_gemm_f64_round_log_nested(False, False, T, DH, T, 1.0, probs, T, T * T, H * T * T, qkv[2 * D:], 3 * D, DH,
                                                 T * 3 * D, None, H, B, y32, DH, T * DH, None, 0, tau, dlog, ws)),
        linear("attn_out", x),
        layer("residual_add_1", vt.VT_LAYER_ADD, x, R, D, reads=2, second=x2),
        layer("layer_norm_2", vt.VT_LAYER_NORM, x2, R, D, eps=1e-5),
        linear("mlp_up", x),
        layer("gelu_tanh", vt.VT_LAYER_GELU_TANH, h4, R, 4 * D),
        linear("mlp_down", h4),
        layer("residual_add_2", vt.VT_LAYER_ADD, x2, R, D, reads=2, second=x),
    ]
    res, per_call = run_stream(b, [(nm, fl, fn) for nm, fl, _, fn in ops])
    res.pop("by_kind")
    rows = []
    for (nm, fl, nbytes, _), ms in zip(ops, per_call):
        row = {"op": nm, "ms": r4(ms)}
        if fl:
            row["TFLOPs"] = round(fl / ms / 1e9, 2)
            row["frac_mfma_peak"] = r4(fl / ms / 1e9 / FP64_MFMA_PEAK_TFLOPS)
        row["GBs_algorithmic"] = round(nbytes / ms / 1e6, 1)
        rows.append(row)
    res["per_op"] = rows
    res["gemm_ms"] = round(sum(ms for (_, fl, _, _), ms in zip(ops, per_call) if fl), 3)
    res["other_ms"] = round(sum(ms for (_, fl, _, _), ms in zip(ops, per_call) if not fl), 3)
    res["workload"] = ("one GPT-2 117M block forward, batch 8 x 1024 tokens, 12 hooked ops: layer norm, QKV, scores (96 x 1024 x 1024 x 64), "
                       "causal softmax over 98304 rows of 1024, probabilities x values (96 x 1024 x 64 x 1024), attention output, residual "
                       "add, layer norm, MLP up, GELU, MLP down, residual add; tau = 1/4 ulp, packed log; operand seeds "
                       "0x240309603000 + 16*3 + 900 + i")
    return {"gpt2_117m_block_forward": res}


def leg_resnet(b: Bench, si):
    """Config 4: the 53 convolutions of ResNet-50 at batch 64, forward, weight gradient and input gradient, tau = 1/4 ulp,
    packed log; per distinct layer shape the roof min(MFMA peak, arithmetic intensity x HBM peak)."""
    vt, torch = b.vt, b.torch
    dev = b.dev
    NB = 64
    layers = resnet50_conv_layers()
    geo = []
    for kind, h, cin, kf, cout, st, pad in layers:
        ho = (h + 2 * pad - kf) // st + 1
        geo.append((kind, vt.Conv2d(NB, h, h, cin, kf, kf, st, st, pad, pad, 1, 1), cin, kf, cout, NB * ho * ho, h, st))
    max_x = max(NB * d.H * d.W * d.C for _, d, *_ in geo[1:])
    max_y = max(g[5] * g[4] for g in geo)
    max_w = max(g[3] * g[3] * g[2] * g[4] for g in geo)
    seeds = {"x_first_layer_U01": si.seed_for(4, 0), "x_post_relu": si.seed_for(4, 1), "dY": si.seed_for(4, 2), "W_unit_normal": si.seed_for(4, 3)}
    x0 = b.up(si.rng(seeds["x_first_layer_U01"]).random(NB * 224 * 224 * 3))                # conv1: U(0,1)
    xbuf = b.up(si.post_relu(max_x, seeds["x_post_relu"]).astype(np.float32).astype(np.float64))   # deeper layers: max(0, N(0,1))
    dybuf = b.up(si.normal(max_y, seeds["dY"], 1e-3))
    wunit = si.normal(max_w, seeds["W_unit_normal"])
    y32 = torch.empty(max(max_y, max_w, max_x), dtype=torch.float32, device=dev)
    dlog = vt.alloc_dense_log(max(max_y, max_w, max_x))
    need = 0
    for _, d, cin, kf, cout, rows, _, _ in geo:
        for mode in (vt.VT_CONV_FORWARD, vt.VT_CONV_WEIGHT_GRAD):
            m, n, k = vt.vt_conv2d_gemm_shape(d, cout, mode)
            need = max(need, vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, m, n, k, 1))
        m, n, k = vt.vt_conv2d_gemm_shape(d, cout, vt.VT_CONV_DATA_GRAD)
        need = max(need, vt.vt_workspace_bytes(vt.VT_OP_CONV_DGRAD_ROUND_LOG, m, n, k, 1))
    ws = vt.alloc_workspace(need)
    tau = 0.25
    # He-normal filters: one buffer per distinct fan-in (the unit normals scaled by sqrt(2 / fan_in)), on the FP32 grid
    wbufs = {}
    for _, d, cin, kf, cout, *_ in geo:
        fan = kf * kf * cin
        if fan not in wbufs:
            wbufs[fan] = b.up((wunit * np.sqrt(2.0 / fan)).astype(np.float32).astype(np.float64))
    fwd, wgr, dgr, meta = [], [], [], []
    for li, (kind, d, cin, kf, cout, rows, h, st) in enumerate(geo):
        fl = 2.0 * rows * cout * kf * kf * cin
        x = x0 if li == 0 else xbuf
        w = wbufs[kf * kf * cin]
        key = f"{kind} {h}x{h}x{cin}->{cout}" + (f" /{st}" if st > 1 else "")
        meta.append((key, fl, rows, cin, kf, cout, NB * h * h * cin))
        if li > 0:      # the network's input needs no gradient
            dgr.append((key, fl, lambda d=d, cout=cout, w=w: vt.vt_conv2d_f64_round_log(
                vt.VT_CONV_DATA_GRAD, d, cout, dybuf, w, None, y32, None, 0, tau, dlog, ws)))
        fwd.append((key, fl, lambda d=d, cout=cout, x=x, w=w: vt.vt_conv2d_f64_round_log(
            vt.VT_CONV_FORWARD, d, cout, x, w, None, y32, None, 0, tau, dlog, ws)))
        wgr.append((key, fl, lambda d=d, cout=cout, x=x: vt.vt_conv2d_f64_round_log(
            vt.VT_CONV_WEIGHT_GRAD, d, cout, x, dybuf, None, y32, None, 0, tau, dlog, ws)))

    def with_roofs(res, mode):
        """by_kind rows get the layer's roof: min(MFMA peak, AI x 8 TB/s) with the algorithmic bytes of the call
        (image + filters or gradients read once in FP64, FP32 outputs and 0.2 B of packed log per output)."""
        seen = {}
        for key, fl, rows, cin, kf, cout, xelems in meta:
            if key in seen or key not in res["by_kind"]:
                continue
            taps = kf * kf * cin
            if mode == "forward":
                nbytes = 8 * (xelems + taps * cout) + 4.2 * rows * cout
            elif mode == "weight_grad":
                nbytes = 8 * (xelems + rows * cout) + 4.2 * taps * cout
            else:
                nbytes = 8 * (rows * cout + taps * cout) + 4.2 * xelems
            ai = fl / nbytes
            roof = min(FP64_MFMA_PEAK_TFLOPS, ai * HBM_PEAK_GBS / 1e3)
            r = res["by_kind"][key]
            r["flop_per_byte"] = round(ai, 1)
            r["roof_TFLOPs"] = round(roof, 1)
            r["frac_roof"] = r4(r["TFLOPs"] / roof)
            seen[key] = True
        return res
    out = {}
    r, _ = run_stream(b, fwd)
    r["workload"] = "config 4: all 53 convolutions of ResNet-50, batch 64, 224 x 224 x 3 input, implicit im2col, tau = 1/4 ulp, packed log"
    out["resnet50_conv_forward"] = with_roofs(r, "forward")
    r, _ = run_stream(b, wgr)
    r["workload"] = "weight gradients of the same 53 layers (deterministic split-K where the plan asks for it)"
    out["resnet50_conv_weight_grad"] = with_roofs(r, "weight_grad")
    r, _ = run_stream(b, dgr)
    r["workload"] = ("input gradients of the 52 layers after the first; flops counted as the forward layer's (a strided layer "
                     "runs one GEMM per stride phase, so the structural zeros of its view are not multiplied)")
    out["resnet50_conv_input_grad"] = with_roofs(r, "input_grad")
    out["resnet50_inputs"] = {"seeds": seeds, "recipe": "first layer U(0,1); deeper layers one max(0, N(0,1)) buffer on the FP32 grid, "
                              "read from its start by every layer; filters He-normal N(0, 2/fan_in); grad-output N(0,1) * 1e-3"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-stream", action="store_true", help="skip the 2^28-element standalone legs (config 5)")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the GPT-2 layer-stream and ResNet-50 convolution legs (configs 3 and 4)")
    ap.add_argument("--cpu-rows", type=int, default=256,
                    help="rows of X the CPU oracle is timed on: per worker process, and for the single-thread figure")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain elementwise kernel over 1 GiB in / 1 GiB out (torch.neg), so that "
                         "HBM byte counters can be scaled against a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    pool = workers = None
    if not args.no_cpu:
        pool, workers = cpu_pool()          # forked before the GPU is initialised; idle until the last leg

    import torch
    import paper_2403_09603_amd as vt
    import synth_inputs as si

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    lib = vt.load_library()
    b = Bench(vt, torch, HipEvents(lib))

    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=b.dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.neg(src, out=dst)
        torch.cuda.synchronize()
        del src, dst

    out, tau, _ = leg_config2(b, args, si)
    torch.cuda.empty_cache()
    out["config1_latency"] = leg_config1(b, si)
    if not args.no_stream:
        out["standalone"] = leg_config5(b, si)
        torch.cuda.empty_cache()
    if not args.no_workloads:
        out["workloads"] = {**leg_gpt2(b, si)}
        torch.cuda.empty_cache()
        out["workloads"].update(leg_gpt2_block(b, si))
        torch.cuda.empty_cache()
        out["workloads"].update(leg_resnet(b, si))
    if pool is not None:
        out["cpu_baseline"] = cpu_baseline(pool, workers, tau, 8192, 3072, 768, args.cpu_rows)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
