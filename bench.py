#!/usr/bin/env python3
"""Benchmark of the attention hot path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: avion_attn_fwd
followed by avion_attn_bwd (its two kernels) on the ViT-B video training batch
(B=32, H=12, N=1568, d=64, non-causal, bf16).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  `value` is algorithmic TFLOP/s of fwd+bwd: 14*B*H*N^2*d flops per step
(fwd 4, bwd 10 including the recomputation of S that the method needs; the second recomputation of
S and dP that the two-kernel backward does for itself is NOT counted).

Timing protocol: an untimed pre-warm (the card idles at a few hundred MHz and needs some tenths of a
second of load to reach its steady clock), W warm-up steps, then exactly K steps between two HIP
events recorded on the launch stream, bracketed by synchronisations.  `ms_per_step` is that event
time / K; the host's wall clock over the same K steps is reported beside it (`ms_per_step_wall`),
and the K-step block is repeated a few times for a median and a minimum (`repeats`).

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
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

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published figure

# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE from rocprofv3 --pmc, scaled by a copy kernel of
# known size); filled in from the summaries under profiles/ -- None until measured.
MEASURED_HBM_BYTES_PER_LAUNCH = {
    # (workload, dtype, kernel) -> (bytes per launch, summary under profiles/ that holds the counters):
    # (2.0 x FETCH_SIZE + 1.0 x WRITE_SIZE) KiB, the factors being what the same counters read for a plain copy of
    # known size.  Measured offline on separate q/k/v tensors with N(0,1) operands; any other run prints null.
    ("vitb_batch", "bf16", "avion_fwd_kernel"): (3.1232e+08, "profiles/vitb_batch_bf16.txt"),
    ("vitb_batch", "bf16", "avion_dq_kernel"): (4.7268e+08, "profiles/vitb_batch_bf16.txt"),
    ("vitb_batch", "bf16", "avion_dkdv_kernel"): (4.7071e+08, "profiles/vitb_batch_bf16.txt"),
    ("vitb_batch", "f16", "avion_fwd_kernel"): (3.1226e+08, "profiles/vitb_batch_f16.txt"),
    ("vitb_batch", "f16", "avion_dq_kernel"): (4.7278e+08, "profiles/vitb_batch_f16.txt"),
    ("vitb_batch", "f16", "avion_dkdv_kernel"): (4.7065e+08, "profiles/vitb_batch_f16.txt"),
    ("vith_d80", "bf16", "avion_fwd_kernel"): (1.3886e+08, "profiles/vith_d80.txt"),
    ("vith_d80", "bf16", "avion_dq_kernel"): (2.1884e+08, "profiles/vith_d80.txt"),
    ("vith_d80", "bf16", "avion_dkdv_kernel"): (2.2160e+08, "profiles/vith_d80.txt"),
    ("vitb_long", "bf16", "avion_fwd_kernel"): (1.5843e+08, "profiles/vitb_long.txt"),
    ("vitb_long", "bf16", "avion_dq_kernel"): (2.4605e+08, "profiles/vitb_long.txt"),
    ("vitb_long", "bf16", "avion_dkdv_kernel"): (2.4492e+08, "profiles/vitb_long.txt"),
}
PREWARM_SECONDS = 0.3


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def event_ms(fn, n, stream):
    """Milliseconds per call of fn over n calls, between two HIP events recorded on `stream`."""
    import torch
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(n):
        fn()
    e1.record(stream)
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / n


def timed(fn, steps, warmup, stream, repeats=3):
    """Median over `repeats` blocks of `steps` calls each (HIP events on `stream`), after `warmup` calls."""
    for _ in range(warmup):
        fn()
    return sorted(event_ms(fn, steps, stream) for _ in range(repeats))[repeats // 2]


def cpu_baseline(w, x, clips):
    """The oracle as it stands, timed on this host on the first `clips` clips of the workload."""
    import oracle
    sub = {n: x[n][:clips] for n in x}
    threads = oracle.max_threads()
    t0 = time.perf_counter()
    oracle.fwd(sub["q"], sub["k"], sub["v"], w.scale)
    oracle.bwd(sub["q"], sub["k"], sub["v"], sub["dO"], w.scale)
    dt = time.perf_counter() - t0
    flops = 14.0 * clips * w.H * w.N * w.N * w.d
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
        "seconds": dt,
        "sample": f"fwd+bwd of the first {clips} of {w.B} clips of the same workload "
                  f"({clips}x{w.H} heads, N={w.N}, d={w.d}), fp64, OpenMP over query rows; "
                  "counted as 14*B*H*N^2*d flops like the GPU value",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="vitb_batch")
    ap.add_argument("--cpu-clips", type=int, default=32)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--operands", choices=("recipe", "zeros", "ones"), default="recipe",
                    help="recipe = the synthetic N(0,1) inputs the metric is quoted on; zeros / ones = constant "
                         "operands, same instruction stream and traffic, to show how much of the time is the "
                         "data-dependent clock throttling of the chip (never the reported configuration)")
    ap.add_argument("--dtype", choices=("bf16", "f16"), default="bf16",
                    help="bf16 = the reported configuration; f16 = the fp16 entry points on the same draws "
                         "rounded to fp16 (the CPU baseline is skipped: it would time the same oracle)")
    ap.add_argument("--layout", choices=("separate", "packed"), default="separate",
                    help="separate = q, k, v as three [B,N,H,d] tensors (the reported configuration); packed = one "
                         "[B,N,3,H,d] tensor through the *_qkvpacked entry points (same kernels, token stride 3*H*d)")
    ap.add_argument("--causal", action="store_true",
                    help="the causal entry points (query i sees keys 0..i) on the same tensors; a diagnostic, the "
                         "value still counts the unmasked 14*B*H*N^2*d flops")
    ap.add_argument("--no-checkpointing", action="store_true",
                    help="skip the extra timing of the step of a layer trained with gradient checkpointing "
                         "(Sec. 4.1 of the paper: the forward runs a second time before the backward), which is "
                         "reported beside the metric and does not change it")
    ap.add_argument("--device-rng", action="store_true",
                    help="draw the N(0,1) inputs with the device's generator instead of the seeded recipe (same "
                         "distribution, seconds instead of minutes for the large small-sequence workloads; for "
                         "profiling runs -- the CPU baseline is skipped)")
    ap.add_argument("--no-other-format", action="store_true", help="skip the fp16 block of a bf16 run")
    ap.add_argument("--no-layernorm", action="store_true", help="skip the layer-normalisation and bias + GELU blocks of the line")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of Q (known size) so that HBM counters of a "
                         "rocprofv3 --pmc run can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on ONE GPU (every (batch, head) pair is an independent problem, so "
                 "more GPUs would each take a share of the batch with no exchange). Run with --gpus 1.")

    import torch
    import synth_inputs as si
    import paper_2309_16669_amd as av

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    if not os.path.exists(av.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    av.load_library()

    w = si.WORKLOADS[args.workload]
    log(f"[bench] generating {w.name} {w.shape} ...")
    f16 = args.dtype == "f16"
    dev = torch.device("cuda:0")
    x = None if args.device_rng else si.make_inputs(w, fmt=args.dtype)

    def up(bits):
        import numpy as np
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(
            torch.float16 if f16 else torch.bfloat16)

    if args.device_rng:
        gen = torch.Generator(device=dev)
        gen.manual_seed(w.seed)
        q, k, v, dO = (torch.randn(w.shape, device=dev, generator=gen, dtype=torch.float32).to(
            torch.float16 if f16 else torch.bfloat16) for _ in range(4))
        if w.k_mul != 1.0:
            k = k * w.k_mul
    else:
        q, k, v, dO = (up(x[n]) for n in ("q", "k", "v", "dO"))
    if args.operands != "recipe":
        for t in (q, k, v, dO):
            t.fill_(0.0 if args.operands == "zeros" else 1.0)
    o = torch.empty_like(q)
    lse = torch.empty((w.B, w.H, w.N), dtype=torch.float32, device=dev)
    dq, dk, dv = (torch.empty_like(q) for _ in range(3))
    ws = torch.empty(av.attn_bwd_workspace_bytes(w.B, w.H, w.N, w.d), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    if args.calibration_copy:
        scratch = torch.empty_like(q)
        for _ in range(3):
            scratch.copy_(q)          # reads and writes q.numel()*2 bytes each
        torch.cuda.synchronize()
        log(f"[bench] calibration copy: {q.numel() * 2} bytes read, {q.numel() * 2} bytes written per launch")

    # the general entry points cover every format / masking / packing; for the reported configuration
    # (bf16, unmasked, separate tensors) they run exactly what avion_attn_fwd / avion_attn_bwd run
    def fwd():
        av.attn_fwd_ex(q, k, v, o, lse, w.scale, args.causal, stream)

    def bwd():
        av.attn_bwd_ex(q, k, v, o, lse, dO, dq, dk, dv, w.scale, ws, args.causal, stream)

    # the phase entry points exist for bf16; for the phase split of an fp16 run they are fed the same
    # bytes viewed as bf16 (same instruction stream and traffic, values irrelevant to a timing)
    as_bf16 = (lambda t: t.view(torch.bfloat16)) if f16 else (lambda t: t)

    def bwd_dq():
        av.attn_bwd_dq(as_bf16(q), as_bf16(k), as_bf16(v), as_bf16(o), lse, as_bf16(dO), as_bf16(dq), w.scale, ws, stream)

    def bwd_dkdv():
        av.attn_bwd_dkdv(as_bf16(q), as_bf16(k), as_bf16(v), lse, as_bf16(dO), as_bf16(dk), as_bf16(dv), w.scale, ws,
                         stream)

    packed = args.layout == "packed"
    if packed:
        qkv = torch.stack((q, k, v), dim=2).contiguous()
        dqkv = torch.empty_like(qkv)

        def fwd():
            av.attn_fwd_ex(qkv, None, None, o, lse, w.scale, args.causal, stream)

        def bwd():
            av.attn_bwd_ex(qkv, None, None, o, lse, dO, dqkv, None, None, w.scale, ws, args.causal, stream)

    def step():
        fwd()
        bwd()

    # untimed pre-warm until the clocks have settled, then W warm-up steps
    t_end = time.perf_counter() + PREWARM_SECONDS
    while time.perf_counter() < t_end:
        for _ in range(10):
            step()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    # whole hot path: exactly K steps between two HIP events on the launch stream (and the host's clock around them)
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(args.steps):
        step()
    e1.record(stream)
    torch.cuda.synchronize()
    ms_wall = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_step = e0.elapsed_time(e1) / args.steps
    repeat_ms = sorted(event_ms(step, args.steps, stream) for _ in range(4))

    # per-phase times, same protocol (median of three K-launch blocks each)
    ms_fwd = timed(fwd, args.steps, 2, stream)
    ms_bwd = timed(bwd, args.steps, 2, stream)
    if packed or f16 or args.causal:
        # these calls have no separate phases: split the backward's time in the proportion of the two
        # kernels of the reported configuration
        a, b = timed(bwd_dq, args.steps, 2, stream), timed(bwd_dkdv, args.steps, 2, stream)
        ms_dq, ms_dkdv = ms_bwd * a / (a + b), ms_bwd * b / (a + b)
    else:
        ms_dq = timed(bwd_dq, args.steps, 2, stream)
        ms_dkdv = timed(bwd_dkdv, args.steps, 2, stream)

    base = w.base
    tf = lambda flops, ms: flops / (ms * 1e-3) / 1e12
    value = tf(14 * base, ms_step)

    # dominant kernel: the key-stationary backward pass (S, dP, dV, dK = 8*base algorithmic flops
    # per launch); the S/dP recomputation inside the dQ pass is the uncredited extra
    dom = {"avion_fwd_kernel": (ms_fwd, 4 * base), "avion_dq_kernel": (ms_dq, 2 * base),
           "avion_dkdv_kernel": (ms_dkdv, 8 * base)}
    dom_name = max(dom, key=lambda n: dom[n][0])
    dom_ms, dom_flops = dom[dom_name]
    achieved = tf(dom_flops, dom_ms)
    # short sequences are bound by memory bandwidth (N/2 flops per byte in the forward, below the chip's
    # ~310): there the whole backward / forward launch is rated by its algorithmic bytes against HBM
    hbm_bound = w.N <= 256
    tensor_bytes = 2.0 * w.B * w.N * w.H * w.d

    out = {
        "metric": "attention fwd+bwd TFLOP/s (N=1568,d=64) and % of MI355X bf16 MFMA peak",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_step_wall": ms_wall,
        "repeats": {"ms_per_step": repeat_ms, "median": repeat_ms[len(repeat_ms) // 2], "min": repeat_ms[0],
                    "note": "further blocks of K steps each, HIP events on the launch stream"},
        "timing": "HIP events on the launch stream around exactly K steps, after an untimed pre-warm of "
                  f"{PREWARM_SECONDS} s and W warm-up steps",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": args.dtype, "data": ("synthetic" if not args.device_rng else "synthetic (device generator)") if args.operands == "recipe" else f"constant operands ({args.operands}), diagnostic only",
        "config": {"workload": f"{w.name}: B={w.B} H={w.H} N={w.N} d={w.d} {'causal' if args.causal else 'non-causal'}, scale={w.scale:g}, "
                               f"Q/K/V/dO ~ N(0,1) {args.dtype}, fwd+bwd" + (", packed [B,N,3,H,d] QKV" if packed else "")
                               + (", CAUSAL variant (diagnostic)" if args.causal else "")},
        "pct_of_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "phases": {
            "fwd": {"ms": ms_fwd, "tflops": tf(4 * base, ms_fwd), "pct_peak": 100 * tf(4 * base, ms_fwd) / PEAK_BF16_TFLOPS},
            "bwd": {"ms": ms_bwd, "tflops": tf(10 * base, ms_bwd), "pct_peak": 100 * tf(10 * base, ms_bwd) / PEAK_BF16_TFLOPS},
            "bwd_dq_kernel_ms": ms_dq, "bwd_dkdv_kernel_ms": ms_dkdv,
            "fwd+bwd": {"ms": ms_step, "tflops": value, "pct_peak": 100 * value / PEAK_BF16_TFLOPS},
        },
        "roofline": {"bound": "mfma", "kernel": dom_name, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
                     "algorithmic_flops_per_launch": dom_flops, "avg_launch_ms": dom_ms},
    }
    if hbm_bound:
        bwd_dom = ms_bwd >= ms_fwd
        nbytes = (8.0 if bwd_dom else 4.0) * tensor_bytes + 4.0 * w.B * w.H * w.N
        rate = nbytes / ((ms_bwd if bwd_dom else ms_fwd) * 1e-3) / 1e9
        out["roofline"] = {"bound": "hbm", "kernel": "backward launch(es)" if bwd_dom else "forward launch",
                           "achieved": rate, "peak": 8000.0, "unit": "GB/s", "frac": rate / 8000.0, "traffic": None,
                           "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": ms_bwd if bwd_dom else ms_fwd,
                           "other": {"fwd_GBps": (4.0 * tensor_bytes) / (ms_fwd * 1e-3) / 1e9,
                                     "bwd_GBps": (8.0 * tensor_bytes) / (ms_bwd * 1e-3) / 1e9}}
    entry = MEASURED_HBM_BYTES_PER_LAUNCH.get((args.workload, args.dtype, dom_name))
    if entry is not None and not packed and not args.causal and args.operands == "recipe":
        out["roofline"]["traffic"] = entry[0]
        out["roofline"]["traffic_source"] = f"rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiled offline: {entry[1]}"
    else:
        out["roofline"]["traffic_source"] = "null: no committed counter summary for this workload / dtype / layout / operands"
    if not args.no_checkpointing:
        def ckpt_step():
            fwd()      # forward pass of the training step (activations dropped)
            fwd()      # recomputation of the layer inside the backward pass
            bwd()
        ms_ckpt = timed(ckpt_step, args.steps, 2, stream)
        out["gradient_checkpointing"] = {
            "ms_per_step": ms_ckpt, "slowdown_vs_plain_step": ms_ckpt / ms_step,
            "note": "fwd + fwd + bwd; still 14*B*H*N^2*d useful flops",
            "tflops_useful": tf(14 * base, ms_ckpt)}
    if not f16 and not args.no_other_format and args.operands == "recipe":
        # the same step on fp16 tensors (the format the paper measured in), values of the same draws
        hq, hk, hv, hdO = (t.to(torch.float16) for t in (q, k, v, dO))
        ho, hdq, hdk, hdv = (torch.empty_like(hq) for _ in range(4))

        def step_f16():
            if packed:
                return
            av.attn_fwd_ex(hq, hk, hv, ho, lse, w.scale, args.causal, stream)
            av.attn_bwd_ex(hq, hk, hv, ho, lse, hdO, hdq, hdk, hdv, w.scale, ws, args.causal, stream)
        if not packed:
            ms_h = timed(step_f16, args.steps, 5, stream)
            out["fp16_entry_points"] = {"ms_per_step": ms_h, "tflops": tf(14 * base, ms_h),
                                        "note": "same step through the fp16 instances; not part of `value`"}
        del hq, hk, hv, hdO, ho, hdq, hdk, hdv
    if not args.no_layernorm:
        # the layer's normalisation on the same tokens ([B*N, H*d], same format): bound by HBM bandwidth;
        # algorithmic bytes: forward reads x and writes y (2 x 2 bytes per element), backward reads x and
        # dy and writes dx (3 x 2), plus two floats per row
        M, D = w.B * w.N, w.H * w.d
        if D % 8 == 0 and D <= 2048:
            xt = torch.randn((M, D), device=dev).to(q.dtype)
            dyt = torch.randn((M, D), device=dev).to(q.dtype)
            gam, bet = torch.ones(D, device=dev), torch.zeros(D, device=dev)
            yt, dxt = torch.empty_like(xt), torch.empty_like(xt)
            mu, rs = torch.empty(M, device=dev), torch.empty(M, device=dev)
            dgam, dbet = torch.empty(D, device=dev), torch.empty(D, device=dev)
            lws = torch.empty(av.layernorm_bwd_workspace_bytes(M, D), dtype=torch.uint8, device=dev)
            ms_lf = timed(lambda: av.layernorm_fwd(xt, gam, bet, yt, mu, rs, 1e-5, stream), args.steps, 5, stream)
            ms_lb = timed(lambda: av.layernorm_bwd(xt, gam, mu, rs, dyt, dxt, dgam, dbet, lws, stream), args.steps, 5, stream)
            bf, bb = 4.0 * M * D + 8.0 * M, 6.0 * M * D + 8.0 * M
            out["layernorm"] = {
                "shape": [M, D], "fwd_ms": ms_lf, "bwd_ms": ms_lb,
                "fwd": {"bound": "hbm", "achieved": bf / (ms_lf * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                        "frac": bf / (ms_lf * 1e-3) / 8e12},
                "bwd": {"bound": "hbm", "achieved": bb / (ms_lb * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                        "frac": bb / (ms_lb * 1e-3) / 8e12},
                "saved_for_backward_bytes_per_token": 2 * D + 8,
                "note": "avion_layernorm_fwd / _bwd on the workload's tokens; not part of `value`"}
            del xt, dyt, yt, dxt
        # the bias + GELU step of the layer's MLP on the same tokens ([B*N, 4*H*d]); algorithmic bytes:
        # forward reads x and writes y, backward reads x and dy and writes dx
        F = 4 * D
        if F % 8 == 0 and F <= 65536:
            xt = (1.5 * torch.randn((M, F), device=dev)).to(q.dtype)
            dyt = torch.randn((M, F), device=dev).to(q.dtype)
            bia, dbia = 0.1 * torch.randn(F, device=dev), torch.empty(F, device=dev)
            yt, dxt = torch.empty_like(xt), torch.empty_like(xt)
            gws = torch.empty(av.bias_gelu_bwd_workspace_bytes(M, F), dtype=torch.uint8, device=dev)
            ms_gf = timed(lambda: av.bias_gelu_fwd(xt, bia, yt, stream), args.steps, 5, stream)
            ms_gb = timed(lambda: av.bias_gelu_bwd(xt, bia, dyt, dxt, dbia, gws, stream), args.steps, 5, stream)
            gf, gb = 4.0 * M * F, 6.0 * M * F
            out["mlp_bias_gelu"] = {
                "shape": [M, F], "fwd_ms": ms_gf, "bwd_ms": ms_gb,
                "fwd": {"bound": "hbm", "achieved": gf / (ms_gf * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                        "frac": gf / (ms_gf * 1e-3) / 8e12},
                "bwd": {"bound": "hbm", "achieved": gb / (ms_gb * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                        "frac": gb / (ms_gb * 1e-3) / 8e12},
                "saved_for_backward_bytes_per_token": 2 * F,
                "note": "avion_bias_gelu_fwd / _bwd on the workload's tokens at the MLP width; not part of `value`"}
            del xt, dyt, yt, dxt
    if not args.no_cpu_baseline and not f16 and not args.device_rng:
        log(f"[bench] timing the CPU oracle on {args.cpu_clips} clips ...")
        out["cpu_baseline"] = cpu_baseline(w, x, min(args.cpu_clips, w.B))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
