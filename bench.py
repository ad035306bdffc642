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
              measured with HIP events on the launch stream inside the timed region
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
    "bytes_per_launch": 25224101198.9,            # mean over the 16 launches t = 0..15 of the counter runs
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
    try:
        digest = kernel_source_digest()
    except OSError:
        return None
    if digest != TRAFFIC["kernel_source_sha256"] or workload_name != TRAFFIC["workload"]:
        return None
    return TRAFFIC["bytes_per_launch"]


def grad_bytes_per_elem(inner: str, grad_dtype: str) -> int:
    g = 4 if grad_dtype == "f32" else 2
    return (24 if inner == "adamw" else 16) + g          # read+write x,m(,v) + read g


def run_gpu(w, steps, warmup, step_waves, outer_waves, outer_variant, extra=False, graph=False, wd_mult=None,
            fused_sync=False, outer_adamw=False):
    import torch

    from paper_2504_18454_amd import Palsgd, make_config, palsgd_layout
    from paper_2504_18454_amd import binding

    binding.lib()                                       # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU is visible; the PALSGD update path runs in HIP kernels only (there is no CPU path)")
    dev = torch.device("cuda:0")
    cfg = make_config(w.K, w.numels, inner=w.inner, grad_dtype=w.grad_dtype, beta1=w.beta1, beta2=w.beta2, eps=w.eps,
                      weight_decay=w.weight_decay, momentum=w.momentum, p=w.p, H=w.H,
                      outer_lr=1e-3 if outer_adamw else w.outer_lr, outer_opt="adamw" if outer_adamw else "sgd",
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
    OV = torch.empty(row, dtype=f, device=dev) if outer_adamw else None   # second moment of OuterOPT = AdamW
    ctx = Palsgd(cfg, X, M, V, G, XG, OM, row, x0=x0, stream=stream, OV=OV)
    if step_waves or outer_waves or outer_variant:
        ctx.palsgd_set_tuning(step_waves, outer_waves, outer_variant)
    torch.cuda.synchronize()

    def one(t, ev=None):
        if ev is not None:
            ev[0].record(stream)
        if fused_sync and (t + 1) % w.H == 0:          # the synchronisation step as one launch
            ctx.palsgd_step_sync(t, w.alpha, w.eta, None, None, stream)
            if ev is not None:
                ev[1].record(stream)
                ev[2].record(stream)
            return True
        ctx.palsgd_step(t, w.alpha, w.eta, None, None, stream)
        if ev is not None:
            ev[1].record(stream)
        if (t + 1) % w.H == 0:
            ctx.palsgd_outer_step(t, stream)
            if ev is not None:
                ev[2].record(stream)
            return True
        return False

    for t in range(warmup):
        one(t)
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
    masks = [ctx.palsgd_draw(t) for t in range(warmup, warmup + steps)]
    synced = []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        synced.append(one(warmup + i, events[i]))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    P = w.P
    gb, mb = grad_bytes_per_elem(w.inner, w.grad_dtype), 12
    all_ms = [events[i][0].elapsed_time(events[i][1]) for i in range(steps)]
    all_bytes = [float(P) * ((K - int(m.sum())) * gb + int(m.sum()) * mb) for m in masks]
    plain = [i for i in range(steps) if not (fused_sync and synced[i])]      # launches of step_kernel
    step_ms, step_bytes = [all_ms[i] for i in plain], [all_bytes[i] for i in plain]
    outer_ms = [events[i][1].elapsed_time(events[i][2]) for i in range(steps) if synced[i]]
    outer_bytes = float(P) * (8 * K + 16 + (8 if outer_adamw else 0))
    total_bytes = sum(all_bytes) + outer_bytes * len(outer_ms)
    fused_ms = [all_ms[i] for i in range(steps) if fused_sync and synced[i]]
    res = dict(
        elapsed=elapsed, updates=float(K) * P * steps, row=row,
        step_kernel_ms_spread=[float(np.percentile(step_ms, q)) for q in (0, 10, 50, 90, 100)],
        step_kernel_ms=float(np.mean(step_ms)), step_kernel_gbps=sum(step_bytes) / (sum(step_ms) * 1e-3) / 1e9,
        step_kernel_bytes=float(np.mean(step_bytes)),
        outer_kernel_ms=float(np.mean(outer_ms)) if outer_ms else None,
        outer_kernel_gbps=(outer_bytes / (np.mean(outer_ms) * 1e-3) / 1e9) if outer_ms else None,
        n_outer=len(outer_ms), mix_fraction=float(np.mean([m.mean() for m in masks])),
        fused_sync_ms=float(np.mean(fused_ms)) if fused_ms else None,
        blended_gbps=total_bytes / elapsed / 1e9,
    )
    torch.cuda.synchronize()
    if graph:
        # the same steps through the device-resident schedule, one captured window of H steps + outer step replayed
        ae = torch.tensor([w.alpha, w.eta], dtype=f, device=dev)
        ctx.palsgd_capturable_begin(warmup + steps, stream)
        torch.cuda.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=stream):
            for _ in range(w.H):
                ctx.palsgd_step_capturable(ae)
            ctx.palsgd_outer_step(0)
        torch.cuda.synchronize()
        windows = max(1, steps // w.H)
        gr.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(windows):
            gr.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ctx.palsgd_capturable_end(stream)
        res["graph"] = dict(windows=windows, ms_per_step=dt / (windows * w.H) * 1e3,
                            value=float(K) * P * windows * w.H / dt)
    if extra:
        # the kernels next to the hot path, each timed alone with events on the launch stream
        def timed(fn, reps=10):
            fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(reps):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / reps
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
        ones, zeros = np.ones(K, np.uint8), np.zeros(K, np.uint8)
        gb_ = grad_bytes_per_elem(w.inner, w.grad_dtype)
        ms = timed(lambda: ctx.palsgd_inner_step(0, w.alpha, None, zeros, stream))
        res["gradient_branch_only"] = dict(ms=ms, gbps=float(P) * K * gb_ / ms / 1e6, bytes_per_elem=gb_)
        if w.p > 0:
            ms = timed(lambda: ctx.palsgd_pseudo_sync(0, w.alpha, w.eta, ones, stream))
            res["mixing_branch_only"] = dict(ms=ms, gbps=float(P) * K * 12 / ms / 1e6, bytes_per_elem=12)
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


def K_bytes(w):
    """Algorithmic bytes per element of a fused synchronisation step with every replica on the gradient branch."""
    return w.K * (grad_bytes_per_elem(w.inner, w.grad_dtype) - 4) + 16 + 4 * w.K


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="gptneo125m_k8")
    ap.add_argument("--step-waves", type=int, default=0, help="resident wavefronts per CU, local update (0 = library's choice)")
    ap.add_argument("--outer-waves", type=int, default=0, help="resident wavefronts per CU, outer step (0 = library's choice)")
    ap.add_argument("--outer-variant", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-decay-1d", action="store_true",
                    help="weight-decay multiplier 0 on one-dimensional tensors (biases, norms): exercises the per-tensor table")
    ap.add_argument("--outer-adamw", action="store_true",
                    help="OuterOPT = AdamW (outer lr 1e-3) instead of the workload's Nesterov momentum")
    ap.add_argument("--fused-sync", action="store_true",
                    help="synchronisation steps as ONE launch (palsgd_step_sync) instead of palsgd_step + palsgd_outer_step")
    ap.add_argument("--graph", action="store_true",
                    help="also time windows of H steps + outer step replayed from one HIP graph (device-resident schedule)")
    ap.add_argument("--extra-kernels", action="store_true",
                    help="also time the DDP warm-up step, gradient-norm clipping and diagnostics kernels")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (K replicas share it); --gpus must be 1. "
              "No multi-GPU figure exists for it.", file=sys.stderr)
        sys.exit(2)
    from paper_2504_18454_amd.workloads import workload
    w = workload(a.workload)
    wd_mult = [0.0 if len(shape) == 1 else 1.0 for _, shape in w.tensors] if a.no_decay_1d else None
    r = run_gpu(w, a.steps, a.warmup, a.step_waves, a.outer_waves, a.outer_variant, a.extra_kernels, a.graph, wd_mult, a.fused_sync, a.outer_adamw)
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
        cpu["one_core"] = {"value": one["value"], "sample": one["sample"]}
        cpu["gpu_over_cpu"] = r["updates"] / r["elapsed"] / cpu["value"]       # context only: the roofline fraction is the measure
    gb = grad_bytes_per_elem(w.inner, w.grad_dtype)
    out = {
        "metric": "replica-param updates/s", "value": r["updates"] / r["elapsed"], "unit": "replica-param updates/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": r["elapsed"] / a.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": a.workload, "K": w.K, "P": w.P, "tensors": len(w.tensors), "inner": w.inner,
                   "grad_dtype": w.grad_dtype, "p": w.p, "H": w.H, "eta": w.eta, "alpha": w.alpha,
                   "outer": "adamw lr 0.001" if a.outer_adamw else f"nesterov lr {w.outer_lr} mu {w.outer_momentum}", "outer_steps_timed": r["n_outer"],
                   "mix_fraction_timed": round(r["mix_fraction"], 4),
                   "weight_decay": "uniform" if not a.no_decay_1d else "per tensor: 0 on 1-D tensors"},
        "hbm_GBps_whole_step": r["blended_gbps"], "hbm_frac_whole_step": r["blended_gbps"] / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": "step_kernel", "achieved": r["step_kernel_gbps"],
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": r["step_kernel_gbps"] / HBM_PEAK_GBPS,
                     "traffic": measured_traffic(a.workload), "bytes_per_launch": r["step_kernel_bytes"], "ms_per_launch": r["step_kernel_ms"],
                     "ms_per_launch_min_p10_p50_p90_max": r["step_kernel_ms_spread"],
                     "bytes_per_elem": {"grad": gb, "mix": 12}},
        "outer_kernel": {"ms_per_launch": r["outer_kernel_ms"], "achieved": r["outer_kernel_gbps"], "unit": "GB/s",
                         "frac": (r["outer_kernel_gbps"] / HBM_PEAK_GBPS) if r["outer_kernel_gbps"] else None,
                         "bytes_per_elem": 8 * w.K + 16 + (8 if a.outer_adamw else 0)},
        "cpu_baseline": cpu,
    }
    if a.fused_sync:
        out["config"]["sync_steps"] = "fused (palsgd_step_sync)"
        out["outer_kernel"] = None
        out["sync_step_kernel"] = {"ms_per_launch": r["fused_sync_ms"],
                                   "bytes_per_elem_all_gradient": K_bytes(w), "unit": "ms"}
    if a.graph:
        out["hip_graph_replay"] = r["graph"]
    if a.extra_kernels:
        out["extra_kernels"] = {k: r[k] for k in ("gradient_branch_only", "mixing_branch_only", "ddp_step", "ddp_step_shared",
                                                  "clip_grad_norm", "clip_mean_grad_norm", "diagnostics") if k in r}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
