#!/usr/bin/env python3
"""Benchmark of the fused attention forward on one MI355X.

One step = one pass of the paper's forward sweep at head dimension 128 (section 4.1,
"Benchmark settings": 16k tokens in total, hidden size 2048 = 16 heads, sequence length
512 ... 16k with batch = 16384 / seqlen), non-causal and causal, once in bf16 (12 launches of
`fa_fwd`) and once in FP8 e4m3 with per-block scales (12 launches of `fa_fwd_fp8`), on inputs
resident in HBM.  FLOPs follow the paper's accounting (4 * N^2 * d * heads * batch, halved when
causal).  Prints one JSON line.
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
# HBM bytes per launch (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc runs of `bench.py --traffic-probe`, scaled
# by what the same counters read for a plain copy of known size), averaged over the launches of the sweep that
# the named kernel serves.  Keyed by kernel name as the library reports it (fa_fwd_kernel_name): a kernel
# that is renamed or re-tiled no longer matches and its traffic is reported as null until it is measured
# again.  Source: profiles/fa_fwd_d128_hbm_traffic.txt.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = {
    "fa_fwd_pingpong_kernel<bf16_tag, 64, 4, false>": 2.966e8,
    "fa_fwd_fp8_async_kernel<128, 128, false, true>": 1.824e8,
}


def attention_flops(B, H, N, d, causal, backward=False):
    """FLOP count by the paper's accounting (section 4.1): 4*N^2*d per head and batch element,
    halved under a causal mask, times 2.5 for the backward pass."""
    f = 4.0 * N * N * d * H * B
    if causal:
        f *= 0.5
    if backward:
        f *= 2.5
    return f


def _cpu_baseline():
    """The fp64 oracle, as it stands, timed on the host cores on a bounded sample."""
    import oracle
    from paper_2407_08608_amd import inputs
    N, d = 8192, HEAD_DIM
    B, H = inputs.benchmark_shape(N, d)
    q, k, v = inputs.qkv(123, B, H, N, d, "bf16")
    q, k, v = (t.double().numpy() for t in (q, k, v))
    t0 = time.perf_counter()
    oracle.attention_fwd(q, k, v, d ** -0.5, False)
    dt = time.perf_counter() - t0
    flops = attention_flops(B, H, N, d, False)
    return {"value": round(flops / dt / 1e12, 4), "unit": "TFLOPs/s", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"the whole seqlen-{N} non-causal point of the sweep (batch {B}, {H} heads), fp64"}


def _hbm_bytes(B, H, N, d, fp8):
    """Compulsory traffic of one forward launch: Q, K, V read and O (16-bit), L (fp32) written once."""
    elems = B * H * N * d
    return (3 * elems + 2 * elems if fp8 else 4 * elems * 2) + 4 * B * H * N


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the per-configuration table outside the headline")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: a plain 256 MiB device copy (calibration) followed by the "
                         "six non-causal bf16 and the six non-causal FP8 forward launches, three times each; "
                         "prints nothing")
    ap.add_argument("--counter-probe", choices=("bwd", "fp8", "fp8_d64", "fp8_d256", "sched4", "sched8", "schedpp"),
                    help="for rocprofv3 --pmc runs: three launches of the bf16 backward (bwd) or of the block-scaled "
                         "FP8 forward (fp8) at seqlen 16k, d = 128, non-causal, or of one forced schedule of the "
                         "fp16 forward at the ablation shape (batch 4, seqlen 8448); prints nothing")
    ap.add_argument("--short-seq-probe", action="store_true",
                    help="instead of the benchmark: seqlen 512 and 1024 at head dimension 128 over a range of batch "
                         "sizes and tile shapes (how the launch time splits into a fixed part and a part per round "
                         "of workgroups); prints one JSON line")
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
    if args.short_seq_probe:
        print(json.dumps(short_seq_probe(torch, binding, inputs, dev)))
        return
    d = HEAD_DIM
    scale = d ** -0.5

    # Inputs resident in HBM before anything is timed.  The FP8 half runs on the same tensors, transformed
    # and quantised once by the library's pre-pass here, outside the timed region (section 3.3 treats the
    # quantisation as fused into the preceding operation; its own rate is in the `extra` table).
    work = []
    signs = inputs.random_signs(1000, d).to(dev)
    for N in SEQLENS:
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(1000 + N, B, H, N, d, "bf16"))
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        work.append(dict(N=N, B=B, H=H, q=q, k=k, v=v, o=o, lse=lse, fp8=(q8, k8, v8, qs, ks, vs)))
    torch.cuda.synchronize()
    stream = torch.cuda.current_stream()

    def launch(w, fp8, causal):
        if fp8:
            binding.fa_fwd_fp8(*w["fp8"], scale, causal, o=w["o"], lse=w["lse"])
        else:
            binding.fa_fwd(w["q"], w["k"], w["v"], scale, causal, o=w["o"], lse=w["lse"])

    def one_step(events=None):
        # 24 launches: the bf16 sweep, then the FP8 sweep; non-causal then causal, seqlen 512 ... 16k
        for fp8 in (False, True):
            for causal in (False, True):
                for w in work:
                    if events is not None:
                        e0 = torch.cuda.Event(enable_timing=True)
                        e1 = torch.cuda.Event(enable_timing=True)
                        e0.record(stream)
                    launch(w, fp8, causal)
                    if events is not None:
                        e1.record(stream)
                        events.append((w["N"], fp8, causal, e0, e1))

    if args.traffic_probe:
        src = torch.empty(256 << 20, device=dev, dtype=torch.uint8).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
            for fp8 in (False, True):
                for w in work:
                    launch(w, fp8, False)
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

    sweep_flops = sum(attention_flops(w["B"], w["H"], w["N"], d, c) for c in (False, True) for w in work)
    ms_per_step = elapsed / args.steps * 1e3
    value = 2 * sweep_flops / (elapsed / args.steps) / 1e12

    # HIP events on the launch stream around every launch: per-launch durations, per-half totals, and the
    # dominant kernel of each half (the kernel the library names for the launch, summed over the step)
    per_point, per_kernel, half_ms = {}, {}, {False: 0.0, True: 0.0}
    for (N, fp8, causal, e0, e1) in events:
        ms = e0.elapsed_time(e1)
        per_point.setdefault((fp8, N, causal), []).append(ms)
        half_ms[fp8] += ms
        B, H = inputs.benchmark_shape(N, d)
        name = binding.fa_fwd_kernel_name(binding.FA_FP8_E4M3 if fp8 else binding.FA_BF16, N, d, causal)
        acc = per_kernel.setdefault((fp8, name), [0.0, 0.0, 0, 0.0])
        acc[0] += ms
        acc[1] += attention_flops(B, H, N, d, causal)
        acc[2] += 1
        acc[3] += _hbm_bytes(B, H, N, d, fp8)

    def roofline_of(fp8):
        (_, name), (ms, flops, n, hbm) = max(((k, v) for k, v in per_kernel.items() if k[0] == fp8),
                                              key=lambda kv: kv[1][0])
        peak = PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS
        achieved = flops / (ms * 1e-3) / 1e12
        traffic = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(name)
        return {"bound": "mfma", "achieved": round(achieved, 1), "peak": peak, "unit": "TFLOP/s",
                "frac": round(achieved / peak, 4), "traffic": traffic, "kernel": name,
                "avg_launch_ms": round(ms / n, 4), "launches": n,
                "algorithmic_flops_per_launch": flops / n, "algorithmic_hbm_bytes_per_launch": hbm / n,
                "share_of_half_time": round(ms / half_ms[fp8], 3)}

    halves = {}
    for fp8, key, peak in ((False, "bf16", PEAK_BF16_TFLOPS), (True, "fp8", PEAK_FP8_TFLOPS)):
        tf = sweep_flops * args.steps / (half_ms[fp8] * 1e-3) / 1e12
        halves[key] = {"tflops": round(tf, 1), "ms_per_step": round(half_ms[fp8] / args.steps, 4),
                       "frac_of_mfma_peak": round(tf / peak, 4), "launches_per_step": 12}

    # per launch: mean and median over the timed steps, and the compulsory HBM traffic as a fraction of the
    # 8 TB/s peak: the short launches sit close to that second roofline
    points = {}
    for (fp8, N, causal), ms_list in sorted(per_point.items()):
        ms = sum(ms_list) / len(ms_list)
        B, H = inputs.benchmark_shape(N, d)
        tf = attention_flops(B, H, N, d, causal) / ms / 1e9
        points[f"{'fp8' if fp8 else 'bf16'}_N{N}_{'causal' if causal else 'full'}"] = {
            "ms": round(ms, 4), "median_ms": round(statistics.median(ms_list), 4), "tflops": round(tf, 1),
            "frac_of_mfma_peak": round(tf / (PEAK_FP8_TFLOPS if fp8 else PEAK_BF16_TFLOPS), 4),
            "hbm_frac": round(_hbm_bytes(B, H, N, d, fp8) / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 3)}

    # the step's working set (257 MiB per shape) is about the size of the last-level cache: one figure with the
    # caches flushed by a 1 GiB fill before every launch, at the shortest shape, where it matters most
    cold = {}
    w = work[0]
    flush = torch.empty(1 << 30, device=dev, dtype=torch.uint8)
    for fp8 in (False, True):
        for causal in (False, True):
            ms_list = []
            for _ in range(10):
                flush.fill_(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                launch(w, fp8, causal)
                e1.record(stream)
                torch.cuda.synchronize()
                ms_list.append(e0.elapsed_time(e1))
            ms = statistics.median(ms_list)
            cold[f"{'fp8' if fp8 else 'bf16'}_N{w['N']}_{'causal' if causal else 'full'}"] = {
                "median_ms": round(ms, 4),
                "tflops": round(attention_flops(w["B"], w["H"], w["N"], d, causal) / ms / 1e9, 1),
                "hbm_frac": round(_hbm_bytes(w["B"], w["H"], w["N"], d, fp8) / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 3)}
    del flush

    out = {
        "metric": "fwd attention TFLOPs/s bf16+fp8, hdim 128, seqlen 512-16k; % of MFMA peak",
        "value": round(value, 2), "unit": "TFLOPs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16+fp8", "data": "synthetic",
        "config": {"workload": "attention fwd, head_dim 128, 16 heads, seqlen {512..16k} x batch 16384/seqlen, "
                               "non-causal + causal: the sweep once in bf16 (fa_fwd) and once in FP8 e4m3 with "
                               "per-block scales (fa_fwd_fp8 on inputs transformed and quantised beforehand): "
                               "24 launches per step; value = FLOPs of both sweeps / wall time of the step"},
        "halves": halves,
        "roofline": roofline_of(False),
        "roofline_fp8": roofline_of(True),
        "points": points,
        "cold_cache": cold,
    }
    if not args.no_extra:
        out["extra"] = extra_table(torch, binding, inputs, dev, work)
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


def short_seq_probe(torch, binding, inputs, dev):
    """Short sequences (bf16, 16 heads, d = 128): launch time against the number of workgroups per CU.
    One row per (seqlen, mask, batch): the library's own choice of kernel and, for comparison, the three
    forced schedules.  256 CUs; a 128-row tile launch has batch * 16 * seqlen / 128 workgroups (causal:
    half, tiles are paired), two of which fit a CU at a time."""
    d, H, rows = 128, 16, {}
    scheds = (("auto", binding.FA_SCHED_AUTO), ("lockstep_4w", binding.FA_SCHED_LOCKSTEP_4W),
              ("lockstep_8w", binding.FA_SCHED_LOCKSTEP_8W), ("pingpong", binding.FA_SCHED_PINGPONG))
    for N in (512, 1024):
        for B in (4, 8, 16, 32, 64, 128):
            q, k, v = (t.to(dev) for t in inputs.qkv(4000 + N + B, B, H, N, d, "bf16"))
            o = torch.empty_like(q)
            lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
            for causal in (False, True):
                row = {}
                for name, sched in scheds:
                    ms = min(_time_call(torch, lambda: binding.fa_fwd_schedule(q, k, v, d ** -0.5, causal, sched,
                                                                               o=o, lse=lse), reps=20, warm=3)
                             for _ in range(2))
                    row[name] = {"us": round(ms * 1e3, 1),
                                 "tflops": round(attention_flops(B, H, N, d, causal) / ms / 1e9, 1),
                                 "hbm_frac": round(_hbm_bytes(B, H, N, d, False) / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S, 3)}
                tiles = B * H * N // 128
                row["workgroups_of_128_rows_per_cu"] = round((tiles // 2 if causal else tiles) / 256, 2)
                rows[f"N{N}_B{B}_{'causal' if causal else 'full'}"] = row
    return rows


def counter_probe(torch, binding, inputs, dev, which):
    """Three launches of one more kernel family for hardware-counter runs."""
    if which.startswith("sched"):
        # the scheduling ablation's shape (section 4.2): batch 4, seqlen 8448, 16 heads, d = 128, fp16, non-causal
        B, H, N, d = 4, 16, 8448, 128
        sched = {"sched4": binding.FA_SCHED_LOCKSTEP_4W, "sched8": binding.FA_SCHED_LOCKSTEP_8W,
                 "schedpp": binding.FA_SCHED_PINGPONG}[which]
        q, k, v = (t.to(dev) for t in inputs.qkv(9, B, H, N, d, "f16"))
        for _ in range(3):
            binding.fa_fwd_schedule(q, k, v, d ** -0.5, False, sched)
        torch.cuda.synchronize()
        return
    N, d = 16384, {"fp8_d64": 64, "fp8_d256": 256}.get(which, 128)
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


def extra_table(torch, binding, inputs, dev, headline_work):
    """Outside the headline: every other row of the path at all six sequence lengths of the sweep (section
    4.1), on seeded inputs: bf16 forward at d = 64 and 256, the FP8 pre-pass and forward at d = 64, 128, 256,
    the bf16 backward at d = 64, 128, 256, and the scheduling ablation at the paper's shape."""
    table = {}

    def tf(B, H, N, d, causal, ms, backward=False):
        return round(attention_flops(B, H, N, d, causal, backward) / ms / 1e9, 1)

    def fwd_rows(d, N, B, H, q, k, v, o, lse):
        for causal in (False, True):
            ms = _time_call(torch, lambda: binding.fa_fwd(q, k, v, d ** -0.5, causal, o=o, lse=lse))
            t = tf(B, H, N, d, causal, ms)
            table[f"fwd_bf16_d{d}_N{N}_{'causal' if causal else 'full'}"] = {
                "ms": round(ms, 4), "tflops": t, "frac_of_mfma_peak": round(t / PEAK_BF16_TFLOPS, 4)}

    def fp8_rows(d, N, B, H, q, k, v, o, lse, tag=""):
        signs = inputs.random_signs(7, d).to(dev)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        ms = _time_call(torch, lambda: binding.fa_fp8_quant_hadamard(q, signs, x8=q8, scales=qs))
        gbps = q.numel() * 3 / ms / 1e6
        table[f"quant_hadamard_d{d}_N{N}{tag}"] = {"ms": round(ms, 4), "GBps": round(gbps, 1),
                                                  "frac_of_hbm_peak": round(gbps * 1e9 / PEAK_HBM_BYTES_PER_S, 3)}
        for causal in (False, True):
            ms = _time_call(torch, lambda: binding.fa_fwd_fp8(q8, k8, v8, qs, ks, vs, d ** -0.5, causal,
                                                              o=o, lse=lse))
            t = tf(B, H, N, d, causal, ms)
            table[f"fwd_fp8_d{d}_N{N}_{'causal' if causal else 'full'}{tag}"] = {
                "ms": round(ms, 4), "tflops": t, "frac_of_mfma_peak": round(t / PEAK_FP8_TFLOPS, 4)}

    def bwd_rows(d, N, B, H, q, k, v, do):
        ws = torch.empty(binding.fa_bwd_workspace_bytes(B, H, N, d), device=dev, dtype=torch.uint8)
        dq, dk, dv = (torch.empty_like(q) for _ in range(3))
        for causal in (False, True):
            o, lse = binding.fa_fwd(q, k, v, d ** -0.5, causal)
            ms = _time_call(torch, lambda: binding.fa_bwd(q, k, v, o, lse, do, d ** -0.5, causal, dq=dq, dk=dk,
                                                          dv=dv, workspace=ws), reps=5)
            t = tf(B, H, N, d, causal, ms, backward=True)
            table[f"bwd_bf16_d{d}_N{N}_{'causal' if causal else 'full'}"] = {
                "ms": round(ms, 4), "tflops": t, "frac_of_mfma_peak": round(t / PEAK_BF16_TFLOPS, 4)}

    for d in (64, 128, 256):
        for N in SEQLENS:
            B, H = inputs.benchmark_shape(N, d)
            if d == HEAD_DIM:
                w = next(w for w in headline_work if w["N"] == N)
                q, k, v, o, lse = w["q"], w["k"], w["v"], w["o"], w["lse"]
            else:
                q, k, v = (t.to(dev) for t in inputs.qkv(2000 + N + d, B, H, N, d, "bf16"))
                o = torch.empty_like(q)
                lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
                fwd_rows(d, N, B, H, q, k, v, o, lse)
            if d != HEAD_DIM:
                fp8_rows(d, N, B, H, q, k, v, o, lse)
            else:  # the d = 128 FP8 forward is in the headline; here only its pre-pass
                signs = inputs.random_signs(7, d).to(dev)
                q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
                ms = _time_call(torch, lambda: binding.fa_fp8_quant_hadamard(q, signs, x8=q8, scales=qs))
                gbps = q.numel() * 3 / ms / 1e6
                table[f"quant_hadamard_d{d}_N{N}"] = {"ms": round(ms, 4), "GBps": round(gbps, 1),
                                                     "frac_of_hbm_peak": round(gbps * 1e9 / PEAK_HBM_BYTES_PER_S, 3)}
            do = inputs.normal_tensor(3000 + N + d, "do", (B, H, N, d), "bf16").to(dev)
            bwd_rows(d, N, B, H, q, k, v, do)
    # FP8 on the heavy-tailed inputs of the paper's error study (section 4.3), on which the running maximum
    # is raised -- and the accumulator rescaled -- far more often
    for d in (128, 256):
        N = 16384
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(7, B, H, N, d, "bf16", heavy_tailed=True))
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        fp8_rows(d, N, B, H, q, k, v, o, lse, tag="_heavy_tailed")
    # scheduling ablation at the paper's shape (section 4.2: batch 4, seqlen 8448, 16 heads, d 128, fp16, non-causal)
    B, H, N, d = 4, 16, 8448, 128
    q, k, v = (t.to(dev) for t in inputs.qkv(9, B, H, N, d, "f16"))
    o = torch.empty_like(q)
    lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
    for name, sched in (("pingpong_async_staging", binding.FA_SCHED_PINGPONG),
                        ("lockstep_8_waves", binding.FA_SCHED_LOCKSTEP_8W),
                        ("lockstep_4_waves_2_workgroups", binding.FA_SCHED_LOCKSTEP_4W)):
        ms = _time_call(torch, lambda: binding.fa_fwd_schedule(q, k, v, d ** -0.5, False, sched, o=o, lse=lse))
        table[f"ablation_f16_b4_s8448_h16_d128_{name}"] = {"ms": round(ms, 4), "tflops": tf(B, H, N, d, False, ms)}
    return table


if __name__ == "__main__":
    main()
