#!/usr/bin/env python3
"""Benchmark of the fused attention forward on one MI355X.

One step = one pass of the paper's forward sweep at head dimension 128 (section 4.1,
"Benchmark settings": 16k tokens in total, hidden size 2048 = 16 heads, sequence length
512 ... 16k with batch = 16384 / seqlen), non-causal and causal: 12 launches of `fa_fwd` on
bf16 inputs resident in HBM.  FLOPs follow the paper's accounting (4 * N^2 * d * heads *
batch, halved when causal).  Prints one JSON line.
"""
import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

SEQLENS = (512, 1024, 2048, 4096, 8192, 16384)
HEAD_DIM = 128
PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak (published)
PEAK_FP8_TFLOPS = 5000.0
PEAK_HBM_BYTES_PER_S = 8.0e12  # published HBM3E bandwidth
# HBM bytes per launch of the dominant kernel (the ping-pong non-causal d=128 kernel, which serves
# seqlen 1k..16k: average over those five shapes), from the rocprofv3 FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/fa_fwd_bf16_d128_hbm_traffic.txt (copy-kernel calibration factors 2.000
# and 1.000): four shapes move 257.3 MiB, seqlen 16k moves 385 MiB.  Algorithmic: 2.695e8 bytes.
TRAFFIC_BYTES_PER_LAUNCH = 2.967e8
DOMINANT_MIN_SEQLEN = 1024  # the launcher uses the 4-wave tile below this (non-causal)


def _cpu_baseline():
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample."""
    import oracle
    from paper_2407_08608_amd import binding, inputs
    N, d = 8192, HEAD_DIM
    B, H = inputs.benchmark_shape(N, d)
    q, k, v = inputs.qkv(123, B, H, N, d, "bf16")
    q, k, v = (t.double().numpy() for t in (q, k, v))
    t0 = time.perf_counter()
    oracle.attention_fwd(q, k, v, d ** -0.5, False)
    dt = time.perf_counter() - t0
    flops = binding.attention_flops(B, H, N, d, False)
    return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOPs/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"the whole seqlen-{N} non-causal point of the sweep (batch {B}, {H} heads), fp64"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the untimed per-config table")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a plain 256 MiB device copy (calibration) followed by the "
                         "six non-causal forward launches, three times each; prints nothing")
    ap.add_argument("--counter-probe", choices=("bwd", "fp8"),
                    help="for rocprofv3 --pmc runs: three launches of the bf16 backward (bwd) or of the block-scaled "
                         "FP8 forward (fp8) at seqlen 16k, d = 128, non-causal; prints nothing")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="instead of the benchmark: the MFMA-only rate of the chip (bf16 and e4m3) on constant and "
                         "on random operand bits; prints one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU; run with --gpus 1 "
                 "(the path shards over batch and heads without communication)")

    import torch
    from paper_2407_08608_amd import binding, inputs

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.mfma_probe:
        print(json.dumps(mfma_probe(torch, binding, inputs, dev)))
        return
    if args.counter_probe:
        counter_probe(torch, binding, inputs, dev, args.counter_probe)
        return
    d = HEAD_DIM
    scale = d ** -0.5

    # inputs resident in HBM before anything is timed
    work = []
    for N in SEQLENS:
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(1000 + N, B, H, N, d, "bf16"))
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        work.append((N, B, H, q, k, v, o, lse))
    stream = torch.cuda.current_stream()

    def one_step(events=None):
        for causal in (False, True):
            for (N, B, H, q, k, v, o, lse) in work:
                if events is not None:
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                binding.fa_fwd(q, k, v, scale, causal, o=o, lse=lse)
                if events is not None:
                    e1.record(stream)
                    events.append((N, causal, e0, e1))

    if args.traffic_probe:
        src = torch.empty(256 << 20, device=dev, dtype=torch.uint8).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
            for (N, B, H, q, k, v, o, lse) in work:
                binding.fa_fwd(q, k, v, scale, False, o=o, lse=lse)
        torch.cuda.synchronize()
        return

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    step_flops = sum(binding.attention_flops(B, H, N, d, c) for c in (False, True) for (N, B, H, *_r) in work)
    ms_per_step = elapsed / args.steps * 1e3
    value = step_flops / (elapsed / args.steps) / 1e12

    # dominant kernel: fa_fwd_pingpong_kernel<bf16, BC=64, P=4, causal=false> (non-causal, seqlen >= 1k;
    # about 60 % of the step's time); its duration comes from HIP events on the launch stream
    dur_ms, flops_dom, n_launch, per_point = 0.0, 0.0, 0, {}
    for (N, causal, e0, e1) in events:
        ms = e0.elapsed_time(e1)
        per_point.setdefault((N, causal), []).append(ms)
        if not causal and N >= DOMINANT_MIN_SEQLEN:
            dur_ms += ms
            n_launch += 1
            B, H = inputs.benchmark_shape(N, d)
            flops_dom += binding.attention_flops(B, H, N, d, False)
    achieved = flops_dom / (dur_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": TRAFFIC_BYTES_PER_LAUNCH,
                "kernel": "fa_fwd_pingpong_kernel<bf16_tag, 64, 4, false>",
                "avg_launch_ms": round(dur_ms / n_launch, 4), "launches": n_launch}

    # per launch: mean and median over the timed steps, and the compulsory HBM traffic (Q, K, V read, O and L
    # written once) as a fraction of the 8 TB/s peak: the short launches sit close to that second roofline
    points = {}
    for (N, causal), ms_list in sorted(per_point.items()):
        ms = sum(ms_list) / len(ms_list)
        B, H = inputs.benchmark_shape(N, d)
        hbm_bytes = 4 * B * H * N * d * 2 + 4 * B * H * N
        points[f"N{N}_{'causal' if causal else 'full'}"] = {
            "ms": round(ms, 4), "median_ms": round(statistics.median(ms_list), 4),
            "tflops": round(binding.attention_flops(B, H, N, d, causal) / ms / 1e9, 1),
            "hbm_frac": round(hbm_bytes / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 3)}

    # the step's working set (257 MiB per shape) is about the size of the last-level cache: one figure with the
    # caches flushed by a 1 GiB fill before every launch, at the shortest shape, where it matters most
    cold = {}
    N, B, H, q, k, v, o, lse = work[0]
    flush = torch.empty(1 << 30, device=dev, dtype=torch.uint8)
    for causal in (False, True):
        ms_list = []
        for _ in range(10):
            flush.fill_(1)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            binding.fa_fwd(q, k, v, scale, causal, o=o, lse=lse)
            e1.record(stream)
            torch.cuda.synchronize()
            ms_list.append(e0.elapsed_time(e1))
        ms = statistics.median(ms_list)
        cold[f"N{N}_{'causal' if causal else 'full'}"] = {
            "median_ms": round(ms, 4), "tflops": round(binding.attention_flops(B, H, N, d, causal) / ms / 1e9, 1),
            "hbm_frac": round((4 * B * H * N * d * 2 + 4 * B * H * N) / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 3)}
    del flush

    out = {
        "metric": "fwd attention TFLOPs/s bf16, hdim 128, seqlen 512-16k (causal + non-causal sweep aggregate)",
        "value": round(value, 2), "unit": "TFLOPs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "attention fwd bf16, head_dim 128, 16 heads, seqlen {512..16k} x batch 16384/seqlen, "
                               "non-causal + causal (12 launches per step)"},
        "roofline": roofline,
        "frac_of_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4),
        "points": points,
        "cold_cache": cold,
    }
    if not args.no_extra:
        out["extra"] = extra_table(torch, binding, inputs, dev)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline()
    print(json.dumps(out))


def mfma_probe(torch, binding, inputs, dev):
    """MFMA-only rate: every wave of a full-chip launch issues independent MFMAs and nothing else.
    `ones` = all operands 1.0; `attention_like` = the bits of N(0,1) draws in bf16, or of the e4m3
    codes of N(0,1) scaled so that the largest magnitude maps to 448.  The drop from `ones` to
    `attention_like` is the clock the chip gives up to the switching activity of real operands."""
    import numpy as np
    out = {"what": "MFMA-only rate, 512 workgroups x 8 waves, TFLOP/s", "peak_bf16": PEAK_BF16_TFLOPS,
           "peak_fp8": PEAK_FP8_TFLOPS}
    x = inputs.normal_tensor(7, "probe", (1 << 16,), "bf16")
    amax = float(x.abs().max())
    operands = {
        ("bf16", "ones"): torch.ones(1 << 16, dtype=torch.bfloat16).view(torch.uint8),
        ("bf16", "attention_like"): x.view(torch.uint8),
        ("fp8", "ones"): torch.full((1 << 16,), 0x38, dtype=torch.uint8),
        ("fp8", "attention_like"): (x.float() * (448.0 / amax)).to(torch.float8_e4m3fn).view(torch.uint8),
    }
    iters = 20000
    for (name, kind), bits in operands.items():
        code = binding.FA_BF16 if name == "bf16" else binding.FA_FP8_E4M3
        t = bits.contiguous().to(dev)
        ms = _time_call(torch, lambda: binding.fa_probe_mfma(t, code, iters), reps=8, warm=4)
        out[f"{name}_{kind}"] = round(binding.fa_probe_mfma_flops(code, iters) / ms / 1e9, 1)
    return out


def counter_probe(torch, binding, inputs, dev, which):
    """Three launches of one more kernel family for hardware-counter runs (seqlen 16k, d = 128, non-causal)."""
    N, d = 16384, 128
    B, H = inputs.benchmark_shape(N, d)
    q, k, v = (t.to(dev) for t in inputs.qkv(7, B, H, N, d, "bf16"))
    if which == "bwd":
        do = inputs.normal_tensor(8, "do", (B, H, N, d), "bf16").to(dev)
        o, lse = binding.fa_fwd(q, k, v, d ** -0.5, False)
        for _ in range(3):
            binding.fa_bwd(q, k, v, o, lse, do, d ** -0.5, False)
    else:
        signs = inputs.random_signs(7, d).to(dev)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        for _ in range(3):
            binding.fa_fwd_fp8(q8, k8, v8, qs, ks, vs, d ** -0.5, False)
    torch.cuda.synchronize()


def _time_call(torch, fn, reps=10, warm=2):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def extra_table(torch, binding, inputs, dev):
    """Outside the timed headline: the other rows of the path at three sequence lengths each."""
    table = {}

    def tf(B, H, N, d, causal, ms, backward=False):
        return round(binding.attention_flops(B, H, N, d, causal, backward) / ms / 1e9, 1)

    for d in (64, 256):  # bf16 forward at the other head dimensions
        for N in (512, 4096, 16384):
            B, H = inputs.benchmark_shape(N, d)
            q, k, v = (torch.randn((B, H, N, d), device=dev, dtype=torch.bfloat16) for _ in range(3))
            o = torch.empty_like(q)
            lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
            for causal in (False, True):
                ms = _time_call(torch, lambda: binding.fa_fwd(q, k, v, d ** -0.5, causal, o=o, lse=lse))
                table[f"fwd_bf16_d{d}_N{N}_{'causal' if causal else 'full'}"] = {
                    "ms": round(ms, 4), "tflops": tf(B, H, N, d, causal, ms)}
    # FP8: pre-pass (HBM-bound) and forward.  Speed rows use N(0,1) inputs like the 16-bit rows; one more
    # row per head dimension uses the heavy-tailed inputs of the paper's error study (section 4.3), on which
    # the running maximum is raised -- and the accumulator rescaled -- far more often.
    for d, N, heavy in [(d, N, False) for d in (64, 128, 256) for N in (512, 4096, 16384)] + [(128, 16384, True),
                                                                                           (256, 16384, True)]:
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(7, B, H, N, d, "bf16", heavy_tailed=heavy))
        tag = "_heavy_tailed" if heavy else ""
        signs = inputs.random_signs(7, d).to(dev)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        ms = _time_call(torch, lambda: binding.fa_fp8_quant_hadamard(q, signs, x8=q8, scales=qs))
        table[f"quant_hadamard_d{d}_N{N}{tag}"] = {"ms": round(ms, 4), "GBps": round(q.numel() * 3 / ms / 1e6, 1)}
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        for causal in (False, True):
            ms = _time_call(torch, lambda: binding.fa_fwd_fp8(q8, k8, v8, qs, ks, vs, d ** -0.5, causal,
                                                              o=o, lse=lse))
            table[f"fwd_fp8_d{d}_N{N}_{'causal' if causal else 'full'}{tag}"] = {
                "ms": round(ms, 4), "tflops": tf(B, H, N, d, causal, ms),
                "frac_of_fp8_peak": round(tf(B, H, N, d, causal, ms) / PEAK_FP8_TFLOPS, 4)}
    # scheduling ablation at the paper's shape (section 4.2: batch 4, seqlen 8448, 16 heads, d 128, fp16, non-causal)
    B, H, N, d = 4, 16, 8448, 128
    q, k, v = (torch.randn((B, H, N, d), device=dev, dtype=torch.float16) for _ in range(3))
    o = torch.empty_like(q)
    lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
    for name, sched in (("pingpong_async_staging", binding.FA_SCHED_PINGPONG),
                        ("lockstep_8_waves", binding.FA_SCHED_LOCKSTEP_8W),
                        ("lockstep_4_waves_2_workgroups", binding.FA_SCHED_LOCKSTEP_4W)):
        ms = _time_call(torch, lambda: binding.fa_fwd_schedule(q, k, v, d ** -0.5, False, sched, o=o, lse=lse))
        table[f"ablation_f16_b4_s8448_h16_d128_{name}"] = {"ms": round(ms, 4), "tflops": tf(B, H, N, d, False, ms)}
    for d, N in ((128, 1024), (128, 4096), (128, 16384), (64, 4096), (64, 16384), (256, 4096), (256, 16384)):  # bf16 backward
        B, H = inputs.benchmark_shape(N, d)
        q, k, v, do = (torch.randn((B, H, N, d), device=dev, dtype=torch.bfloat16) for _ in range(4))
        ws = torch.empty(binding.fa_bwd_workspace_bytes(B, H, N, d), device=dev, dtype=torch.uint8)
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        for causal in (False, True):
            o, lse = binding.fa_fwd(q, k, v, d ** -0.5, causal)
            ms = _time_call(torch, lambda: binding.fa_bwd(q, k, v, o, lse, do, d ** -0.5, causal, dq=dq, dk=dk,
                                                          dv=dv, workspace=ws), reps=5)
            table[f"bwd_bf16_d{d}_N{N}_{'causal' if causal else 'full'}"] = {
                "ms": round(ms, 4), "tflops": tf(B, H, N, d, causal, ms, backward=True)}
    return table


if __name__ == "__main__":
    main()
