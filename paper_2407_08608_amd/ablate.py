"""Measurement aid: what each part of the forward's block costs on the GPU, and the clock the chip runs at.

Builds variants of libfa_mi355.so in which fa_fwd_fp8.hip is compiled with FA_ABLATE=1..4 (one part of
fa_fwd_fp8_kernel's block removed; results wrong on purpose) or with FA_PHASE_TRACE (shader-clock stamps at
the phase boundaries of 32 blocks of one workgroup), into csrc/_build/ablate/, and times the block-scaled
FP8 forward at head dimension 128 with each of them on the seeded N(0,1) inputs of the benchmark.

    python -m paper_2407_08608_amd.ablate --build        # on the CPU (hipcc cross-compiles)
    python -m paper_2407_08608_amd.ablate --run          # on the GPU; prints a table
    python -m paper_2407_08608_amd.ablate --clock        # on the GPU; shader-clock cycles and clock per kernel

--clock uses one more library, every kernel file compiled with FA_CLOCK_SPAN (ClockSpan in fa_device.h): the
main kernels record their first entry and last exit stamp on one CU, and cycles over wall time is the clock
the chip granted that kernel.

The library itself is never built with these switches.
"""
import argparse
import ctypes
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
OUT = os.path.join(HERE, "csrc", "_build", "ablate")  # git-ignored, travels to the GPU machine with the tree
# FA_STAGED_TILE8: the eight-wave tile with register staging, the kernel these switches instrument (the library
# runs the same block arithmetic in fa_fwd_fp8_async_kernel, whose staging bypasses the registers)
VARIANTS = {"full": ["-DFA_STAGED_TILE8"], "no_exponentials": ["-DFA_STAGED_TILE8", "-DFA_ABLATE=1"],
            "no_lds_reads_second_gemm": ["-DFA_STAGED_TILE8", "-DFA_ABLATE=2"],
            "no_second_gemm": ["-DFA_STAGED_TILE8", "-DFA_ABLATE=3"],
            "no_softmax_arithmetic": ["-DFA_STAGED_TILE8", "-DFA_ABLATE=4"],
            "phase_trace": ["-DFA_STAGED_TILE8", "-DFA_PHASE_TRACE"], "library": []}
# the bf16 ping-pong kernel (fa_fwd.hip)
VARIANTS_16 = {"full": [], "no_exponentials": ["-DFA_ABLATE_PP=1"], "no_v_operand_reads": ["-DFA_ABLATE_PP=2"],
               "no_k_operand_reads": ["-DFA_ABLATE_PP=3"], "no_softmax_arithmetic": ["-DFA_ABLATE_PP=4"]}


def build():
    from . import build as fa_build
    fa_build.build(verbose=False)  # the other objects come from the regular build
    os.makedirs(OUT, exist_ok=True)
    others = [os.path.join(fa_build.OBJ, f) for f in sorted(os.listdir(fa_build.OBJ))
              if f.endswith(".hip.o") and f != "fa_fwd_fp8.hip.o"]
    for name, flags in VARIANTS.items():
        obj = os.path.join(OUT, f"fa_fwd_fp8_{name}.o")
        subprocess.run([fa_build.HIPCC, *fa_build.FLAGS, *flags, "-c", os.path.join(fa_build.CSRC, "fa_fwd_fp8.hip"),
                        "-o", obj], check=True, stderr=subprocess.DEVNULL)
        subprocess.run([fa_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o",
                        os.path.join(OUT, f"libfa_{name}.so"), obj, *others], check=True)
        print("built", name, file=sys.stderr)
    others = [os.path.join(fa_build.OBJ, f) for f in sorted(os.listdir(fa_build.OBJ))
              if f.endswith(".hip.o") and f != "fa_fwd.hip.o"]
    for name, flags in VARIANTS_16.items():
        obj = os.path.join(OUT, f"fa_fwd_{name}.o")
        subprocess.run([fa_build.HIPCC, *fa_build.FLAGS, *flags, "-c", os.path.join(fa_build.CSRC, "fa_fwd.hip"),
                        "-o", obj], check=True, stderr=subprocess.DEVNULL)
        subprocess.run([fa_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o",
                        os.path.join(OUT, f"libfa16_{name}.so"), obj, *others], check=True)
        print("built bf16", name, file=sys.stderr)
    objs = []
    for src in sorted(f for f in os.listdir(fa_build.CSRC) if f.endswith(".hip")):
        obj = os.path.join(OUT, f"clock_span_{src}.o")
        subprocess.run([fa_build.HIPCC, *fa_build.FLAGS, *fa_build.EXTRA_FLAGS.get(src, []), "-DFA_CLOCK_SPAN", "-c",
                        os.path.join(fa_build.CSRC, src), "-o", obj], check=True, stderr=subprocess.DEVNULL)
        objs.append(obj)
    subprocess.run([fa_build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o",
                    os.path.join(OUT, "libfa_clock_span.so"), *objs], check=True)
    print("built clock_span", file=sys.stderr)


def run(seqlens):
    import numpy as np
    import torch
    from . import binding, inputs
    d, dev = 128, torch.device("cuda:0")
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    libs = {}
    for name in VARIANTS:
        L = ctypes.CDLL(os.path.join(OUT, f"libfa_{name}.so"))
        L.fa_fwd_fp8.argtypes = [vp] * 8 + [ci] * 5 + [cf, ci, vp]
        L.fa_fwd_fp8.restype = ci
        libs[name] = L
    st = torch.cuda.current_stream().cuda_stream
    for N in seqlens:
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(1000 + N, B, H, N, d, "bf16"))
        signs = inputs.random_signs(1000, d).to(dev)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        flops = 4.0 * N * N * d * H * B
        for causal in (0, 1):
            row = []
            for name, L in libs.items():
                def call():
                    r = L.fa_fwd_fp8(q8.data_ptr(), k8.data_ptr(), v8.data_ptr(), qs.data_ptr(), ks.data_ptr(),
                                     vs.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d, 128, d ** -0.5, causal, st)
                    assert r == 0
                for _ in range(5):
                    call()
                torch.cuda.synchronize()
                best = 1e9
                for _ in range(2):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(20):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    best = min(best, e0.elapsed_time(e1) / 20)
                row.append(f"{name} {flops * (0.5 if causal else 1) / best / 1e9:7.1f}")
            print(f"N={N} causal={causal} nominal TFLOPs/s: " + "  ".join(row), flush=True)
    # phase trace of the eight-wave kernel at the last sequence length, non-causal (workgroup 300, blocks 60..91)
    L = libs["phase_trace"]
    L.fa_fwd_fp8(q8.data_ptr(), k8.data_ptr(), v8.data_ptr(), qs.data_ptr(), ks.data_ptr(), vs.data_ptr(), o.data_ptr(),
                 lse.data_ptr(), B, H, N, d, 128, d ** -0.5, 0, st)
    torch.cuda.synchronize()
    buf = np.zeros(8 * 32 * 8, dtype=np.int64)
    L.fa_debug_read_phase_trace(buf.ctypes.data_as(vp))
    tr = buf.reshape(8, 32, 8)
    names = ["scores", "mask+max+reference", "P~ (scale, exp2, sum, e4m3)", "products", "tile stores", "barrier wait"]
    print("phase trace (shader-clock cycles, mean over blocks 64..87 of workgroup 300; waves w and w+4 share a SIMD):")
    for w in range(8):
        r = tr[w]
        seg = (r[:, 1:7] - r[:, 0:6])[4:28].mean(axis=0)
        print(f"  wave {w}: period {np.diff(r[:, 0])[4:28].mean():6.0f}   " + "   ".join(f"{n} {x:5.0f}" for n, x in zip(names, seg)))


def run16(seqlens):
    """The bf16 forward at head dimension 128 (ping-pong kernel from 1024 keys on) with each variant."""
    import torch
    from . import inputs
    d, dev = 128, torch.device("cuda:0")
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    libs = {}
    for name in VARIANTS_16:
        L = ctypes.CDLL(os.path.join(OUT, f"libfa16_{name}.so"))
        L.fa_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_fwd.restype = ci
        libs[name] = L
    st = torch.cuda.current_stream().cuda_stream
    for N in seqlens:
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(1000 + N, B, H, N, d, "bf16"))
        o = torch.empty_like(q)
        lse = torch.empty((B, H, N), device=dev, dtype=torch.float32)
        flops = 4.0 * N * N * d * H * B
        for causal in (0, 1):
            row = []
            for name, L in libs.items():
                def call():
                    r = L.fa_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d,
                                 d ** -0.5, causal, 1, st)
                    assert r == 0
                for _ in range(5):
                    call()
                torch.cuda.synchronize()
                best = 1e9
                for _ in range(2):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(20):
                        call()
                    e1.record()
                    torch.cuda.synchronize()
                    best = min(best, e0.elapsed_time(e1) / 20)
                row.append(f"{name} {flops * (0.5 if causal else 1) / best / 1e9:7.1f}")
            print(f"bf16 N={N} causal={causal} nominal TFLOPs/s: " + "  ".join(row), flush=True)


def clock(N):
    """Cycles on one CU, wall time and the resulting clock of the main kernels at N keys (benchmark shapes)."""
    import numpy as np
    import torch
    from . import binding, inputs
    dev = torch.device("cuda:0")
    vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    L = ctypes.CDLL(os.path.join(OUT, "libfa_clock_span.so"))
    L.fa_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, cf, ci, ci, vp]
    L.fa_fwd_fp8.argtypes = [vp] * 8 + [ci] * 5 + [cf, ci, vp]
    L.fa_bwd.argtypes = [vp] * 9 + [vp, ctypes.c_size_t] + [ci] * 4 + [cf, ci, ci, vp]
    for f in (L.fa_fwd, L.fa_fwd_fp8, L.fa_bwd):
        f.restype = ci
    st = torch.cuda.current_stream().cuda_stream
    reps = 5
    print(f"{reps} launches back to back after 10 warm-up launches; cycles: first entry to last exit stamp on one CU")
    for d in (128, 64, 256):
        B, H = inputs.benchmark_shape(N, d)
        q, k, v = (t.to(dev) for t in inputs.qkv(1000 + N, B, H, N, d, "bf16"))
        do = inputs.qkv(2000 + N, B, H, N, d, "bf16")[0].to(dev)
        signs = inputs.random_signs(1000, d).to(dev)
        q8, qs = binding.fa_fp8_quant_hadamard(q, signs)
        k8, ks = binding.fa_fp8_quant_hadamard(k, signs)
        v8, vs = binding.fa_fp8_quant_hadamard(v, None)
        o, lse = binding.fa_fwd(q, k, v, d ** -0.5, False)
        o8 = torch.empty_like(q)
        dq, dk, dv = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        ws = torch.empty(B * H * N, device=dev, dtype=torch.float32)
        for causal in (0, 1):
            if causal:
                o, lse = binding.fa_fwd(q, k, v, d ** -0.5, True)
            calls = {
                "fwd bf16": (L.fa_debug_clock_span_fwd, 4.0, lambda: L.fa_fwd(
                    q.data_ptr(), k.data_ptr(), v.data_ptr(), o8.data_ptr(), lse.data_ptr(), B, H, N, d, d ** -0.5,
                    causal, binding.FA_BF16, st)),
                "fwd fp8": (L.fa_debug_clock_span_fwd_fp8, 4.0, lambda: L.fa_fwd_fp8(
                    q8.data_ptr(), k8.data_ptr(), v8.data_ptr(), qs.data_ptr(), ks.data_ptr(), vs.data_ptr(),
                    o8.data_ptr(), lse.data_ptr(), B, H, N, d, 128, d ** -0.5, causal, st)),
                "bwd bf16": (L.fa_debug_clock_span_bwd, 10.0, lambda: L.fa_bwd(
                    q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), do.data_ptr(),
                    dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), ws.data_ptr(), ws.numel() * 4, B, H, N, d,
                    d ** -0.5, causal, binding.FA_BF16, st)),
            }
            for what, (reader, flop_factor, call) in calls.items():
                if what == "fwd fp8":
                    lse_keep = lse.clone()  # the FP8 forward overwrites L, which the backward reads
                span = np.zeros(2, dtype=np.uint64)
                reader.argtypes = [vp]
                for _ in range(10):
                    assert call() == 0
                assert reader(span.ctypes.data_as(vp)) == 0
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    assert call() == 0
                e1.record()
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                assert reader(span.ctypes.data_as(vp)) == 0
                cycles = int(span[1]) - int(span[0])
                flops = flop_factor * N * N * d * H * B * (0.5 if causal else 1) * reps
                print(f"d={d:3d} N={N} causal={causal} {what}: {ms / reps:7.4f} ms per launch  {flops / ms / 1e9:7.1f} "
                      f"nominal TFLOPs/s  {cycles / reps:10.0f} cycles per launch  clock {cycles / ms / 1e6:5.3f} GHz",
                      flush=True)
                if what == "fwd fp8":
                    lse.copy_(lse_keep)


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--build", action="store_true")
    ap.add_argument("--run", action="store_true")
    ap.add_argument("--clock", action="store_true")
    ap.add_argument("--seqlens", default="4096,16384")
    a = ap.parse_args()
    if a.build:
        build()
    if a.run:
        run16([int(x) for x in a.seqlens.split(",")])
        run([int(x) for x in a.seqlens.split(",")])
    if a.clock:
        clock(int(a.seqlens.split(",")[-1]))
