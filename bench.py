#!/usr/bin/env python3
"""Benchmark of the encoder-layer hot path on one MI355X.

A step is one forward + one backward pass of the whole layer (every kernel of the
path) over one batch of the seeded synthetic workload, inputs resident in HBM.
Prints ONE JSON line: tokens/s (B*T per step), the roofline figures of the kernel
class that takes the most time (measured with HIP events on the launch stream in a
second pass of the same steps), and the fp64 CPU oracle timed on the host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

roofline.traffic cannot be measured from inside the process (the HBM byte counters need
rocprofv3 around it); it is read from the committed summary profiles/layer_<workload>_hbm_traffic.txt
of two counter runs of this same command (written by `python -m paper_2201_12465_amd.profile_summary
traffic ...`, which also gives the commands) and is null when no summary exists for the workload.
`--copy-calibration` runs only the library's plain copy kernel over a known size: the kernel those
counters are scaled by.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}   # MI355X dense MFMA peaks
PEAK_HBM_GBS = 8000.0
MFMA_CLASSES = ("gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd", "attn_bwd")
COPY_BYTES = 256 << 20


def stored_traffic(workload: str, kernel_class: str):
    """HBM bytes per launch of one kernel class from the committed counter summary, or None."""
    path = os.path.join(ROOT, "profiles", f"layer_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        f = line.split()
        if len(f) >= 4 and f[0] == "traffic" and f[1] == kernel_class and f[2] == "bytes_per_launch":
            return float(f[3]), os.path.relpath(path, ROOT)
    return None, None


def copy_run(b, torch, stream, launches: int):
    """`launches` plain copies of COPY_BYTES; returns GB/s of read + written bytes."""
    src = torch.ones(COPY_BYTES // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    T = b.test_lib()   # the probes live in the test build of the library; the timed layer runs on the product
    b.check(T.fl_test_copy(src.data_ptr(), dst.data_ptr(), COPY_BYTES, stream), T)
    e0.record()
    for _ in range(launches):
        b.check(T.fl_test_copy(src.data_ptr(), dst.data_ptr(), COPY_BYTES, stream), T)
    e1.record()
    torch.cuda.synchronize()
    assert bool((dst[:: 1 << 16] == 1).all())
    return 2.0 * COPY_BYTES * launches / (e0.elapsed_time(e1) * 1e-3) / 1e9


def mfma_probe_run(b, torch, stream, dtype: str, launches: int = 3):
    """TFLOP/s of an MFMA-only loop (operands in registers) of the workload's type on this GPU."""
    import ctypes
    wgs, iters = 256 * 16, 1000 if dtype == "bf16" else 250   # four wavefronts per SIMD, about 2 ms per launch
    sink = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    flops = ctypes.c_double(0.0)
    dt = b.FL_BF16 if dtype == "bf16" else b.FL_F32
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    T = b.test_lib()
    b.check(T.fl_test_mfma_probe(dt, wgs, iters, sink.data_ptr(), ctypes.byref(flops), stream), T)
    e0.record()
    for _ in range(launches):
        b.check(T.fl_test_mfma_probe(dt, wgs, iters, sink.data_ptr(), ctypes.byref(flops), stream), T)
    e1.record()
    torch.cuda.synchronize()
    return flops.value * launches / (e0.elapsed_time(e1) * 1e-3) / 1e12


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg3_bert_base_bf16")
    ap.add_argument("--causal", action="store_true", help="the workload with the causal attention mask added")
    ap.add_argument("--dropout", type=float, default=0.0,
                    help="training mode: this rate at all four dropout sites, a new seed every step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true",
                    help="skip the second, event-instrumented pass (used under rocprofv3)")
    ap.add_argument("--no-deferred-join", action="store_true",
                    help="multi-layer workloads: every layer's backward joins the side stream before it returns")
    ap.add_argument("--no-grad-overlap", action="store_true",
                    help="run the parameter-gradient kernels in order on the main stream instead of beside "
                         "the input-gradient chain (every kernel then runs alone: the mode for kernel traces)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only 5 launches of the plain copy kernel over 256 MiB (counter calibration)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2201_12465_amd import binding as b
    from workloads import CONFIGS, layer_flops, make_inputs, make_stack_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    b.lib()   # fails loudly if the HIP library has not been built
    if a.copy_calibration:
        gbs = copy_run(b, torch, torch.cuda.current_stream().cuda_stream, 4)
        print(json.dumps({"copy_kernel": "copy_kernel", "bytes_read": COPY_BYTES, "bytes_written": COPY_BYTES,
                          "launches": 5, "gbs": gbs}))
        return 0
    b.set_grad_overlap(not a.no_grad_overlap)
    cfg = CONFIGS[a.workload]
    if a.causal:
        cfg = cfg.with_(name=cfg.name + "+causal", causal=True)
    if a.dropout > 0:
        cfg = cfg.with_(name=cfg.name + f"+dropout{a.dropout:g}")
    tdt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    dev = lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda().to(tdt).contiguous()
    if cfg.layers > 1:
        inp = make_stack_inputs(cfg, seed=0)
        plist = inp["params"]
    else:
        inp = make_inputs(cfg, seed=0)
        plist = [inp["params"]]
    nl = len(plist)
    P = [{k: dev(v) for k, v in p.items()} for p in plist]
    G = [{k: torch.empty_like(v) for k, v in p.items()} for p in P]
    acts = [dev(inp["X"])] + [torch.empty(inp["X"].shape, dtype=tdt, device="cuda") for _ in range(nl)]
    grads = [torch.empty(inp["X"].shape, dtype=tdt, device="cuda") for _ in range(nl)] + [dev(inp["dY"])]
    L = torch.from_numpy(inp["lengths"]).cuda() if inp["lengths"] is not None else None
    layers = [b.Layer(cfg.B, cfg.T, cfg.D, cfg.H, cfg.F, cfg.act, cfg.norm, cfg.dtype, cfg.eps, cfg.causal)
              for _ in range(nl)]
    stream = torch.cuda.current_stream().cuda_stream

    seeds = iter(range(1, 1 << 30))

    def step():
        for l in range(nl):
            if a.dropout > 0:
                layers[l].set_dropout(a.dropout, a.dropout, next(seeds))
            layers[l].forward(P[l], acts[l], L, cfg.B, cfg.T, acts[l + 1], stream)
        for l in reversed(range(nl)):
            layers[l].backward(P[l], grads[l + 1], grads[l], G[l], stream)
        if deferred:   # the parameter gradients of the whole stack are complete after these
            for l in range(nl):
                layers[l].join(stream)

    # a stack joins its layers' side-stream work once, after the last backward, instead of after every layer
    deferred = nl > 1 and not a.no_deferred_join
    for ly in layers:
        ly.set_deferred_join(deferred)
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    warm_stats = b.alloc_stats()
    # Exactly a.steps timed steps between two device synchronisations.  Events on the stream cut them into up
    # to 10 blocks without stalling the queue: ms_per_step (and `value`) is the MEDIAN block; the fastest
    # block and the wall-clock mean over all steps go beside it.
    nblocks = max(1, min(10, a.steps // 2)) if a.steps >= 10 else 1
    sizes = [a.steps // nblocks + (1 if i < a.steps % nblocks else 0) for i in range(nblocks)]
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(nblocks + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks[0].record()
    for i, n in enumerate(sizes):
        for _ in range(n):
            step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    end_stats = b.alloc_stats()
    block_ms = [marks[i].elapsed_time(marks[i + 1]) / n for i, n in enumerate(sizes)]
    ms_per_step = float(np.median(block_ms))
    secs = ms_per_step * 1e-3 * a.steps      # the median block's rate over the a.steps steps
    tokens = cfg.B * cfg.T
    fl = layer_flops(cfg, inp["lengths"])
    flops_step = fl["fwd_bwd"] * nl

    out = {
        "metric": "layer fwd+bwd tokens/s", "value": tokens * a.steps / secs, "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_min": min(block_ms), "ms_per_step_wall_mean": wall / a.steps * 1e3,
        "timed_blocks": nblocks,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "T": cfg.T, "d_model": cfg.D, "heads": cfg.H, "d_ffn": cfg.F,
                   "act": cfg.act, "norm": cfg.norm, "layers": nl,
                   "mask": ("key-padding lengths" if L is not None else "none") + (" + causal" if cfg.causal else "")},
        "tflops_algorithmic": flops_step / (secs / a.steps) / 1e12,
        "valid_tokens_per_s": (float(np.sum(inp["lengths"])) if L is not None else tokens) * a.steps / secs,
        "device_mallocs_in_timed_region": end_stats["backing_mallocs"] - warm_stats["backing_mallocs"],
        "grad_overlap": not a.no_grad_overlap,
    }

    # ---- per-kernel-class timing: same steps again, every launch bracketed by HIP events on `stream`
    if not a.no_kernel_timing:
        # with the side stream off, so that each kernel runs alone and its duration is its own
        ksteps = min(a.steps, 20)
        b.set_grad_overlap(False)
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(ksteps):
            step()
        torch.cuda.synchronize()
        out["ms_per_step_without_grad_overlap"] = (time.perf_counter() - t0) / ksteps * 1e3
        b.prof_enable("all")
        for _ in range(ksteps):
            step()
        torch.cuda.synchronize()
        prof = b.prof_collect()
        b.prof_enable(None)
        b.set_grad_overlap(not a.no_grad_overlap)
        mask_scale = fl["fwd_attn"] / (4.0 * cfg.D * cfg.T * tokens)      # 1 without a mask
        kernels = {}
        for name, e in prof.items():
            flops = e["flops"] * (mask_scale if name.startswith("attn") else 1.0)   # library counts dense attention
            us = e["total_ms"] * 1e3 / e["launches"]    # event bracket: the kernel plus a few microseconds
            kernels[name] = {"launches_per_step": e["launches"] / ksteps, "avg_us": us,
                             "ms_per_step": e["total_ms"] / ksteps,
                             "tflops": flops / e["total_ms"] / 1e9 if flops else None,
                             "gbs": e["bytes"] / e["total_ms"] / 1e6}
        # what a bracket with no kernel in it reads (an upper bound of the part of avg_us that is not the kernel)
        out["event_bracket_empty_us"] = next(iter(prof.values()))["empty_bracket_ms"] * 1e3 if prof else None
        dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
        k = kernels[dom]
        if dom in MFMA_CLASSES:
            peak = PEAK_TFLOPS[cfg.dtype]
            roof = {"kernel": dom, "bound": "mfma", "achieved": k["tflops"], "peak": peak, "unit": "TFLOP/s",
                    "frac": k["tflops"] / peak, "traffic": None, "avg_us": k["avg_us"]}
        else:
            roof = {"kernel": dom, "bound": "hbm", "achieved": k["gbs"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": k["gbs"] / PEAK_HBM_GBS, "traffic": None, "avg_us": k["avg_us"]}
        roof["traffic"], src = stored_traffic(cfg.name, dom)
        if src:
            roof["traffic_source"] = src
            roof["algorithmic_bytes_per_launch"] = k["gbs"] * 1e9 * k["avg_us"] * 1e-6
        out["roofline"] = roof
        out["kernels"] = kernels
        out["hbm_copy_gbs"] = copy_run(b, torch, stream, 10)   # what a plain copy reaches on this GPU
        out["mfma_probe_tflops"] = mfma_probe_run(b, torch, stream, cfg.dtype)   # and an MFMA-only loop
        # the same fraction against what the probes reach on this GPU (the datasheet peak stays in `frac`)
        measured = out["mfma_probe_tflops"] if roof["bound"] == "mfma" else out["hbm_copy_gbs"]
        roof["peak_measured"] = measured
        roof["frac_of_measured"] = roof["achieved"] / measured

    # ---- the fused optimizer step (NOT part of `value`: the metric is the layer's forward + backward)
    if not a.no_kernel_timing:
        names = list(P[0].keys())
        ne = [P[0][k].numel() for k in names]
        ms_ = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in ne]
        vs_ = [torch.zeros(n, dtype=torch.float32, device="cuda") for n in ne]
        pcopy = [P[0][k].clone() for k in names]          # the benchmark's own parameters stay untouched
        gl = [G[0][k] for k in names]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for it in range(3):
            b.opt_step("adam", cfg.dtype, pcopy, gl, ms_, vs_, ne, stream, lr=1e-4, step=it + 1)
        e0.record()
        for it in range(20):
            b.opt_step("adam", cfg.dtype, pcopy, gl, ms_, vs_, ne, stream, lr=1e-4, step=it + 4)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / 20 * 1e3
        esz = 4 if cfg.dtype == "f32" else 2
        by = sum(ne) * (3 * esz + 16)                      # read p, g, m, v; write p, m, v
        out["optimizer_step"] = {"kind": "adam", "tensors": len(ne), "elements": sum(ne), "avg_us": us,
                                 "gbs": by / us / 1e3, "frac_of_hbm_peak": by / us / 1e3 / PEAK_HBM_GBS}

    # ---- the fp64 CPU oracle on the host cores (a reported baseline, not a target)
    if not a.no_cpu_baseline:
        from oracle import oracle as orc
        threads = len(os.sched_getaffinity(0))
        try:
            from threadpoolctl import threadpool_info
            blas = [i["num_threads"] for i in threadpool_info() if i.get("user_api") == "blas"]
            if blas:
                threads = max(blas)
        except Exception:
            pass
        kw = dict(heads=cfg.H, act=cfg.act, norm=cfg.norm, eps=cfg.eps, causal=cfg.causal)
        if a.dropout > 0:   # the oracle pays for drawing the masks, as the kernels do
            from oracle import dropout as odr
        # bounded sample: the first sequences of the batch, sized for roughly 10-30 s of CPU work
        nb = cfg.B if nl == 1 and cfg.M <= 4096 else max(1, min(cfg.B, 4096 // cfg.T))
        sl = slice(0, nb)
        lens = inp["lengths"][sl] if L is not None else None
        t0 = time.perf_counter()
        reps = 0
        while reps < 1 or (time.perf_counter() - t0 < 10.0 and reps < 20):
            if a.dropout > 0:
                kw["masks"] = odr.layer_masks(nb, cfg.T, cfg.D, cfg.H, cfg.F, a.dropout, a.dropout, reps + 1)
            orc.layer_forward_backward(plist[0], inp["X"][sl], inp["dY"][sl], lens, **kw)
            reps += 1
        cs = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": nb * cfg.T / cs, "unit": "tokens/s", "cores": threads, "kind": "oracle",
                               "sample": f"{nb} of {cfg.B} sequences, one layer fwd+bwd, fp64 numpy, "
                                         f"mean of {reps} run(s), {cs:.2f} s each"}
    print(json.dumps(out))
    for ly in layers:
        ly.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
