#!/usr/bin/env python3
"""Benchmark of the PALSGD parameter-update path on one MI355X.

A step is one iteration of Alg. 1 for all K replicas: the fused local update (gradient
step or pseudo-synchronization step per replica, as the seeded branch draws decide) and,
when (t+1) mod H == 0, the outer step.  Inputs are synthetic, seeded and already resident
in HBM when the timed region starts.  Prints ONE JSON line:

  value       K*P*steps / elapsed: replica-parameter updates per second
  roofline    the fused local-update kernel against the HBM peak: algorithmic bytes per
              launch (26 B per replica-element on the AdamW/bf16 gradient branch, 28 fp32,
              20 SGD-momentum, 12 on the mixing branch) over its mean launch duration,
              measured with HIP events on the launch stream inside the timed region (one event per launch
              boundary: a launch's duration runs to the start of the next)
  cpu_baseline the CPU oracle timed on a bounded slice of the same workload

    python bench.py [--gpus 1] [--steps 256] [--warmup 64] [--workload gptneo125m_k8]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of step_kernel from two rocprofv3 counter runs (FETCH_SIZE, WRITE_SIZE, each scaled by
# what it reads for the 1 GiB set-up copy); summary in profiles/gptneo125m_k8_hbm_counters.txt.  The figure
# holds for one kernel source only: it is reported as null as soon as the code of step_kernel and its helpers
# (csrc/device_common.h and csrc/step_kernel.h, comments and white space aside) differs from the files the
# counters were taken with.
TRAFFIC = {
    "workload": "gptneo125m_k8",
    "kernel_source_sha256": "2b4b472afa213a9d7fc1d8fd969690649f8cde613eeda7b322a7d303d24f09fa",
    "bytes_per_launch": 25224111946.2,            # mean over the 16 launches t = 0..15 of the counter runs
    "algorithmic_bytes_same_launches": 25224565440.0,
}


def kernel_source_digest(csrc=None):
    """SHA-256 of the code of step_kernel and its helpers (the two headers that hold them) with comments and
    white space removed: a change of that kernel's code changes it, a change of wording, of other kernels or
    of host code does not."""
    import hashlib
    import re
    csrc = csrc or os.path.join(ROOT, "paper_2504_18454_amd", "csrc")
    text = "".join(open(os.path.join(csrc, name), "r").read() for name in ("device_common.h", "step_kernel.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    text = re.sub(r"\s+", "", text)
    return hashlib.sha256(text.encode()).hexdigest()


def measured_traffic(workload_name):
    """(counter bytes per launch, algorithmic bytes of the launches the counters saw), or (None, None) when the
    counters were taken with another kernel source or workload."""
    try:
        digest = kernel_source_digest()
    except OSError:
        return None, None
    if digest != TRAFFIC["kernel_source_sha256"] or workload_name != TRAFFIC["workload"]:
        return None, None
    return TRAFFIC["bytes_per_launch"], TRAFFIC["algorithmic_bytes_same_launches"]


def grad_bytes_per_elem(inner: str, grad_dtype: str) -> int:
    g = 4 if grad_dtype == "f32" else 2
    return (24 if inner == "adamw" else 16) + g          # read+write x,m(,v) + read g


def run_gpu(w, steps, warmup, reps, step_waves, outer_waves, outer_variant, extra=False, graph=False, wd_mult=None,
            fused_sync=False):
    import torch

    from paper_2504_18454_amd import Palsgd, make_config, palsgd_layout
    from paper_2504_18454_amd import binding

    binding.lib()                                       # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU is visible; the PALSGD update path runs in HIP kernels only (there is no CPU path)")
    dev = torch.device("cuda:0")
    cfg = make_config(w.K, w.numels, inner=w.inner, grad_dtype=w.grad_dtype, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                      weight_decay=w.weight_decay, momentum=w.momentum, p=w.p, H=w.H, outer_lr=w.outer_lr,
                      outer_momentum=w.outer_momentum, outer_nesterov=w.outer_nesterov, seed=w.seed, wd_mult=wd_mult)
    row, offs = palsgd_layout(cfg)
    K = w.K
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.seed)
    f = torch.float32
    x0 = torch.empty(row, dtype=f, device=dev).normal_(0.0, 0.02, generator=gen)
    pad = torch.ones(row, dtype=torch.bool, device=dev)
    for o, n in zip(offs, w.numels):
        pad[o:o + n] = False
    pad_idx = pad.nonzero().flatten()
    del pad
    x0.index_fill_(0, pad_idx, 0.0)
    X = torch.empty((K, row), dtype=f, device=dev)
    M = torch.empty((K, row), dtype=f, device=dev)
    V = torch.empty((K, row), dtype=f, device=dev) if w.inner == "adamw" else None
    XG = torch.empty(row, dtype=f, device=dev)
    OM = torch.empty(row, dtype=f, device=dev)
    G = torch.empty((K, row), dtype=f if w.grad_dtype == "f32" else torch.bfloat16, device=dev)
    # gradients of 0.5|x - c|^2 at x0 plus noise, generated once (their values do not affect cost)
    c = torch.empty(row, dtype=f, device=dev).normal_(0.0, 1.0, generator=gen)
    for k in range(K):
        g = torch.empty(row, dtype=f, device=dev).normal_(0.0, w.sigma, generator=gen)
        g.add_(x0).sub_(c)
        g.index_fill_(0, pad_idx, 0.0)
        G[k].copy_(g)
    del g, c
    # one plain device copy of exactly 1 GiB in and 1 GiB out, outside the timed region: the
    # reference dispatch that scales the HBM byte counters of a profiler run of this command
    cal_src = torch.zeros(1 << 28, dtype=f, device=dev)
    cal_dst = torch.empty_like(cal_src)
    cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    stream = torch.cuda.Stream(device=dev)
    ctx = Palsgd(cfg, X, M, V, G, XG, OM, row, x0=x0, stream=stream)
    if step_waves or outer_waves or outer_variant:
        ctx.palsgd_set_tuning(step_waves, outer_waves, outer_variant)
    torch.cuda.synchronize()

    def one(t, marks=None):
        """Step t of Alg. 1.  marks: list that receives one HIP event per launch boundary of this step, recorded on the
        launch stream: before the local update, and on a synchronisation step between it and the outer step.  The
        next step's first event (or the window's closing one) ends the last launch, so a launch costs one event
        record, not two (on the 8.4M-parameter workload three records per step cost 5 % of the step)."""
        def mark():
            if marks is not None:
                e = torch.cuda.Event(enable_timing=True)
                e.record(stream)
                marks.append(e)
        mark()
        if fused_sync and (t + 1) % w.H == 0:          # the synchronisation step as one launch
            ctx.palsgd_step_sync(t, w.alpha, w.eta, None, None, stream)
            return True
        ctx.palsgd_step(t, w.alpha, w.eta, None, None, stream)
        if (t + 1) % w.H == 0:
            mark()
            ctx.palsgd_outer_step(t, stream)
            return True
        return False

    for t in range(warmup):
        one(t)
    torch.cuda.synchronize()
    # `reps` timed windows of exactly `steps` consecutive steps of Alg. 1 each (t runs on from window to window, so
    # synchronisation steps fall where (t+1) mod H = 0 puts them); the reported figure is the median window
    P = w.P
    gb, mb = grad_bytes_per_elem(w.inner, w.grad_dtype), 12
    outer_bytes = float(P) * (8 * K + 16)
    windows, outer_ms, fused_ms = [], [], []
    t_next = warmup
    for _ in range(reps):
        marks = []
        masks = [ctx.palsgd_draw(t) for t in range(t_next, t_next + steps)]
        synced = []
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            synced.append(one(t_next + i, marks))
        closing = torch.cuda.Event(enable_timing=True)
        closing.record(stream)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        t_next += steps
        marks.append(closing)
        by = [float(P) * ((K - int(m.sum())) * gb + int(m.sum()) * mb) for m in masks]
        n_sync = sum(synced)
        all_ms, all_bytes = [], []                       # this window's launches of step_kernel
        j = 0                                            # index of the event that opens step i
        for i in range(steps):
            ms = marks[j].elapsed_time(marks[j + 1])     # the local update (or the fused synchronisation step)
            if fused_sync and synced[i]:
                fused_ms.append(ms)
            else:
                all_ms.append(ms)
                all_bytes.append(by[i])
            j += 1
            if synced[i] and not fused_sync:
                outer_ms.append(marks[j].elapsed_time(marks[j + 1]))
                j += 1
        assert j == len(marks) - 1
        windows.append(dict(elapsed=elapsed, n_outer=n_sync, bytes=sum(by) + outer_bytes * n_sync,
                            mix=float(np.mean([m.mean() for m in masks])), step_ms=all_ms, step_bytes=all_bytes))
    order = sorted(range(reps), key=lambda r: windows[r]["elapsed"])
    med = windows[order[len(order) // 2]]
    all_ms, all_bytes = med["step_ms"], med["step_bytes"]   # the roofline figure is that of the window `value` is quoted on

    # every kernel of the path alone, right after the windows, with events on the launch stream around each launch:
    # the outer step (after an untimed local update, as in Alg. 1), the fused synchronisation step, and each branch
    # of the local update with the branch forced for all K workers
    def each(fn, n=6, before=None):
        # all launches are enqueued without a host wait in between, so the device is still busy with the previous
        # one while the host prepares the next and the events bracket kernel time, not host latency
        pairs = []
        for _ in range(n + 1):
            if before is not None:
                before()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            fn()
            b.record(stream)
            pairs.append((a, b))
        torch.cuda.synchronize()
        return [a.elapsed_time(b) for a, b in pairs[1:]]   # the first launch of a kernel is not counted

    def kern(ms, bytes_per_elem):
        m = float(np.median(ms))
        gbps = float(P) * bytes_per_elem / m / 1e6
        return dict(ms_per_launch=m, ms_min_max=[float(min(ms)), float(max(ms))], launches=len(ms), achieved=gbps,
                    unit="GB/s", frac=gbps / HBM_PEAK_GBPS, bytes_per_elem=bytes_per_elem)

    ones, zeros = np.ones(K, np.uint8), np.zeros(K, np.uint8)
    local = lambda: ctx.palsgd_step(t_next, w.alpha, w.eta, None, None, stream)
    alone_outer = each(lambda: ctx.palsgd_outer_step(t_next, stream), before=local)
    alone_sync = each(lambda: ctx.palsgd_step_sync(t_next, w.alpha, w.eta, None, zeros, stream))
    alone_grad = each(lambda: ctx.palsgd_inner_step(t_next, w.alpha, None, zeros, stream))
    alone_mix = each(lambda: ctx.palsgd_pseudo_sync(t_next, w.alpha, w.eta, ones, stream)) if w.p > 0 else None
    step_ms_mean = float(np.mean(all_ms))
    outer_med = float(np.median(outer_ms + alone_outer))
    bytes_mean = float(np.mean(all_bytes))
    res = dict(
        elapsed=med["elapsed"], updates=float(K) * P * steps, row=row, reps=reps, median_window=order[len(order) // 2],
        window_ms_per_step=[windows[r]["elapsed"] / steps * 1e3 for r in order],
        window_outer_steps=[windows[r]["n_outer"] for r in order],
        n_outer=med["n_outer"], mix_fraction=med["mix"], blended_gbps=med["bytes"] / med["elapsed"] / 1e9,
        step_kernel_ms_spread=[float(np.percentile(all_ms, q)) for q in (0, 10, 50, 90, 100)],
        step_kernel_ms=step_ms_mean, step_kernel_gbps=sum(all_bytes) / (sum(all_ms) * 1e-3) / 1e9,
        step_kernel_bytes=bytes_mean, step_kernel_launches=len(all_ms),
        outer=kern(outer_ms + alone_outer, 8 * K + 16), outer_in_windows=len(outer_ms),
        sync_step=kern(alone_sync + fused_ms, K * (gb - 4) + 16 + 4 * K),
        grad_only=kern(alone_grad, K * gb), mix_only=kern(alone_mix, K * mb) if alone_mix else None,
        # one step of Alg. 1 with the synchronisation step's share: kernel time from the events, bytes from the
        # timed launches' own branch mix
        amortised_ms=step_ms_mean + outer_med / w.H,
        amortised_gbps=(bytes_mean + outer_bytes / w.H) / ((step_ms_mean + outer_med / w.H) * 1e-3) / 1e9,
    )
    t_after = t_next + 1
    torch.cuda.synchronize()
    if graph:
        # the same steps through the device-resident schedule, one captured window of H steps + outer step replayed
        ae = torch.tensor([w.alpha, w.eta], dtype=f, device=dev)
        ctx.palsgd_capturable_begin(t_after, stream)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=stream):
            for _ in range(w.H):
                ctx.palsgd_step_capturable(ae)
            ctx.palsgd_outer_step(0)
        torch.cuda.synchronize()
        n_win = max(1, steps // w.H)
        gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(n_win):
            gr.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.palsgd_capturable_end(stream)
        res["graph"] = dict(windows=n_win, ms_per_step=dt / (n_win * w.H) * 1e3,
                            value=float(K) * P * n_win * w.H / dt)
    if extra:
        # the kernels next to the hot path, each timed alone with events on the launch stream
        def timed(fn, n=10):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(n):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / n
        gB = 4 if w.grad_dtype == "f32" else 2
        state = 12 if w.inner == "adamw" else 8
        out2 = torch.empty(2, dtype=f, device=dev)
        norms = torch.empty(K, dtype=f, device=dev)
        ms = timed(lambda: ctx.palsgd_clip_grad_norm(1.0, norms, stream))
        res["clip_grad_norm"] = dict(ms=ms, gbps=float(P) * K * gB / ms / 1e6, bytes_per_elem=K * gB)
        ms = timed(lambda: ctx.palsgd_clip_mean_grad_norm(1.0, None, norms, stream))
        res["clip_mean_grad_norm"] = dict(ms=ms, gbps=float(P) * K * gB / ms / 1e6, bytes_per_elem=K * gB)
        ms = timed(lambda: ctx.palsgd_diagnostics(out2, stream))
        res["diagnostics"] = dict(ms=ms, gbps=float(P) * (4 * K + 4) / ms / 1e6, bytes_per_elem=4 * K + 4)
        ctx.palsgd_outer_step(0, stream)                # workers identical again, as the DDP step requires
        tau0 = max(ctx.palsgd_get_state()[0])
        ctx.palsgd_set_state([tau0] * K, ctx.palsgd_get_state()[1])
        ddp_b = K * gB + state + 4 + 4 * K + (state - 4)  # read K gradients + x, m(, v); write XG, K rows of x, one of m(, v)
        ms = timed(lambda: ctx.palsgd_ddp_step(0, w.alpha, None, stream))
        res["ddp_step"] = dict(ms=ms, gbps=float(P) * ddp_b / ms / 1e6, bytes_per_elem=ddp_b)
        ddp_s = ddp_b - 4 * K                            # the model kept once (XG): no row stores
        ms = timed(lambda: ctx.palsgd_ddp_step_shared(0, w.alpha, None, stream))
        res["ddp_step_shared"] = dict(ms=ms, gbps=float(P) * ddp_s / ms / 1e6, bytes_per_elem=ddp_s)
    ctx.palsgd_destroy()
    return res


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return None


def run_cpu_baseline(w, slice_div=2, threads=None):
    """The oracle, as it stands, on the first 1/slice_div of every replica row for H+1 steps."""
    import oracle
    from paper_2504_18454_amd.workloads import flat_layout, to_bf16_bits

    if threads is None:
        threads = max(1, min(int(os.environ.get("OMP_NUM_THREADS", "0") or 0) or (os.cpu_count() or 1),
                             os.cpu_count() or 1))
    oracle.set_threads(threads)
    offs, row = flat_layout(w.numels)
    n = max(64, row // slice_div // 64 * 64)
    rng = np.random.default_rng(w.seed)
    x0 = (0.02 * rng.standard_normal(n, dtype=np.float32)).astype(np.float32)
    st = oracle.OracleState(w.K, x0, [0], [n], inner=w.inner, grad_dtype=w.grad_dtype, beta1=w.beta1, beta2=w.beta2,
                            eps=w.eps, weight_decay=w.weight_decay, momentum=w.momentum, p=w.p, H=w.H,
                            outer_lr=w.outer_lr, outer_momentum=w.outer_momentum, outer_nesterov=w.outer_nesterov,
                            seed=w.seed)
    for k in range(w.K):
        g = (x0 - rng.standard_normal(n, dtype=np.float32) + np.float32(w.sigma) * rng.standard_normal(n, dtype=np.float32))
        st.G[k] = g if w.grad_dtype == "f32" else to_bf16_bits(g)
    steps = w.H + 1
    st.iteration(0, w.alpha, w.eta)                      # touch every page once
    t0 = time.perf_counter()
    for t in range(1, steps + 1):
        st.iteration(t, w.alpha, w.eta)
    dt = time.perf_counter() - t0
    return dict(value=float(w.K) * n * steps / dt, unit="replica-param updates/s", cores=threads, kind="oracle",
                sample=f"first {n} elements of each of the K={w.K} replica rows (1/{slice_div} of the row), "
                       f"{steps} steps incl. one outer step, {dt:.1f} s")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--reps", type=int, default=5, help="timed windows of --steps steps each; the median one is reported")
    ap.add_argument("--workload", default="gptneo125m_k8")
    ap.add_argument("--step-waves", type=int, default=0, help="resident wavefronts per CU, local update (0 = library's choice)")
    ap.add_argument("--outer-waves", type=int, default=0, help="resident wavefronts per CU, outer step (0 = library's choice)")
    ap.add_argument("--outer-variant", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decay-1d", action="store_true",
                    help="weight-decay multiplier 0 on one-dimensional tensors (biases, norms): exercises the per-tensor table")
    ap.add_argument("--fused-sync", action="store_true",
                    help="synchronisation steps as ONE launch (palsgd_step_sync) instead of palsgd_step + palsgd_outer_step")
    ap.add_argument("--graph", action="store_true",
                    help="also time windows of H steps + outer step replayed from one HIP graph (device-resident schedule)")
    ap.add_argument("--extra-kernels", action="store_true",
                    help="also time the DDP warm-up step, gradient-norm clipping and diagnostics kernels")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this library runs on ONE GPU (K replicas share it); --gpus must be 1. "
              "No multi-GPU figure exists for it.", file=sys.stderr)
        sys.exit(2)
    if a.reps < 1 or a.steps < 1:
        sys.exit("bench.py: --steps and --reps must be >= 1")
    from paper_2504_18454_amd.workloads import workload
    w = workload(a.workload)
    wd_mult = [0.0 if len(shape) == 1 else 1.0 for _, shape in w.tensors] if a.no_decay_1d else None
    r = run_gpu(w, a.steps, a.warmup, a.reps, a.step_waves, a.outer_waves, a.outer_variant, a.extra_kernels, a.graph,
                wd_mult, a.fused_sync)
    cpu = None
    if not a.no_cpu_baseline:
        # bounded sample: about K * 62M * (H+1) element updates for the all-threads leg whatever the workload
        # (the benchmark configuration: half of every row), 1/32 of that for the one-core leg
        budget = 8 * 62206080 * 65
        div = 2
        while w.K * (w.P // div) * (w.H + 1) > budget:
            div *= 2
        cpu = run_cpu_baseline(w, slice_div=div)
        one = run_cpu_baseline(w, slice_div=32 * div, threads=1)  # the same loop on one core, smaller slice
        cpu["cpu_model"] = cpu_model()
        cpu["one_core"] = {"value": one["value"], "sample": one["sample"]}
        cpu["gpu_over_cpu"] = r["updates"] / r["elapsed"] / cpu["value"]       # context only: the roofline fraction is the measure
    gb = grad_bytes_per_elem(w.inner, w.grad_dtype)
    traffic, traffic_alg = measured_traffic(a.workload)
    out = {
        "metric": "replica-param updates/s", "value": r["updates"] / r["elapsed"], "unit": "replica-param updates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["elapsed"] / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": a.workload, "K": w.K, "P": w.P, "tensors": len(w.tensors), "inner": w.inner,
                   "grad_dtype": w.grad_dtype, "p": w.p, "H": w.H, "eta": w.eta, "alpha": w.alpha,
                   "outer": f"nesterov lr {w.outer_lr} mu {w.outer_momentum}", "outer_steps_timed": r["n_outer"],
                   "mix_fraction_timed": round(r["mix_fraction"], 4),
                   "weight_decay": "uniform" if not a.no_decay_1d else "per tensor: 0 on 1-D tensors"},
        # value and ms_per_step are the MEDIAN of `reps` timed windows of `steps` steps each (sorted list beside it)
        # (median_window: its index in time order, from 0; the roofline figures are those of its launches)
        "reps": r["reps"], "median_window": r["median_window"], "ms_per_step_of_each_window_sorted": r["window_ms_per_step"],
        "outer_steps_in_each_window_sorted": r["window_outer_steps"],
        "hbm_GBps_whole_step": r["blended_gbps"], "hbm_frac_whole_step": r["blended_gbps"] / HBM_PEAK_GBPS,
        # one step of Alg. 1 with 1/H of a synchronisation step's outer launch, from kernel event times
        "step_with_outer_share": {"ms": r["amortised_ms"], "achieved": r["amortised_gbps"], "unit": "GB/s",
                                  "frac": r["amortised_gbps"] / HBM_PEAK_GBPS},
        "roofline": {"bound": "hbm", "kernel": "step_kernel", "achieved": r["step_kernel_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": r["step_kernel_gbps"] / HBM_PEAK_GBPS,
                     # counter bytes per launch of the counter runs, the algorithmic bytes of those same launches, their
                     # ratio (the launches timed here have their own branch mix, hence their own bytes_per_launch)
                     "traffic": traffic, "traffic_algorithmic_same_launches": traffic_alg,
                     "traffic_ratio": (traffic / traffic_alg) if traffic else None,
                     "bytes_per_launch": r["step_kernel_bytes"], "ms_per_launch": r["step_kernel_ms"],
                     "launches": r["step_kernel_launches"],
                     "ms_per_launch_min_p10_p50_p90_max": r["step_kernel_ms_spread"],
                     "bytes_per_elem": {"grad": gb, "mix": 12}},
        # the outer step (outer_kernel_walk): launches inside the windows plus six timed alone right after them
        "outer_kernel": dict(r["outer"], launches_in_windows=r["outer_in_windows"]),
        # each kernel of the path alone (median of six launches, HIP events on the launch stream)
        "branch_kernels": {"gradient_branch_only": r["grad_only"], "mixing_branch_only": r["mix_only"],
                           "fused_sync_step": r["sync_step"]},
        "cpu_baseline": cpu,
    }
    if a.fused_sync:
        out["config"]["sync_steps"] = "fused (palsgd_step_sync)"
    if a.graph:
        out["hip_graph_replay"] = r["graph"]
    if a.extra_kernels:
        out["extra_kernels"] = {k: r[k] for k in ("ddp_step", "ddp_step_shared", "clip_grad_norm", "clip_mean_grad_norm",
                                                  "diagnostics") if k in r}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
