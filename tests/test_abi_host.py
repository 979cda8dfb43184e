"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import bench
from paper_2407_08608_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fa_mi355.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    names = _declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_status_strings():
    assert binding.status_string(0) == "ok"
    seen = {binding.status_string(s) for s in range(8)}
    assert len(seen) == 8
    assert binding.status_string(99) == "unknown status"


def test_fa_fwd_rejects_bad_arguments_without_launching():
    L = binding.lib()
    p = ctypes.c_void_p(0x1000)  # never dereferenced: validation fails first
    ok = dict(B=1, H=1, N=16, d=64, scale=0.125, causal=0, dtype=binding.FA_BF16)

    def call(q=p, k=p, v=p, o=p, lse=p, **kw):
        a = dict(ok, **kw)
        return L.fa_fwd(q, k, v, o, lse, a["B"], a["H"], a["N"], a["d"], a["scale"], a["causal"], a["dtype"], None)

    assert call(q=None) == 1 and call(lse=None) == 1
    assert call(N=0) == 2 and call(B=-1) == 2 and call(scale=0.0) == 2 and call(scale=float("nan")) == 2
    assert call(causal=2) == 2
    assert call(dtype=7) == 3
    assert call(d=96) == 4
    assert call(dtype=binding.FA_F32, d=128, q=ctypes.c_void_p(0x1008)) == 5
    assert call(k=ctypes.c_void_p(0x1004)) == 5
    # documented size limits: B*H*N below 2^31 rows, 4*N*d below 0x7ff00000 bytes per head
    assert call(B=2048, H=1024, N=1024) == 2
    assert call(N=0x7ff00000 // (4 * 128) + 1, d=128) == 4 and call(N=0x7ff00000 // (4 * 64) + 1, d=64) == 4


def test_fp8_and_bwd_entry_points_validate():
    L = binding.lib()
    p = ctypes.c_void_p(0x1000)
    assert L.fa_fwd_fp8(p, p, p, p, p, p, p, p, 1, 1, 16, 128, 64, 0.1, 0, None) == 4  # block_rows != 128
    assert L.fa_fwd_fp8(p, p, p, None, p, p, p, p, 1, 1, 16, 128, 128, 0.1, 0, None) == 1
    assert L.fa_fp8_quant_hadamard(p, binding.FA_FP8_E4M3, p, p, 1, 1, 16, 128, 128, None, 0, None) == 4
    assert L.fa_fp8_quant_hadamard(p, 9, p, p, 1, 1, 16, 128, 128, None, 0, None) == 3
    assert L.fa_fp8_quant_hadamard(p, binding.FA_BF16, p, p, 1, 1, 0, 128, 128, None, 0, None) == 2
    assert L.fa_bwd_workspace_bytes(1, 1, 16, 96, binding.FA_BF16) == 0  # unsupported head dim
    assert L.fa_bwd_workspace_bytes(1, 1, 16, 64, binding.FA_BF16) == 64
    assert L.fa_bwd_workspace_bytes(1, 1, 16, 256, binding.FA_F32) == 0  # unsupported dtype
    args = [p] * 10 + [0, 1, 1, 16, 256, 0.1, 0, binding.FA_F32, None]
    assert L.fa_bwd(*args) == 4
    args = [p] * 9 + [None, 0, 1, 1, 16, 128, 0.1, 0, binding.FA_BF16, None]
    assert L.fa_bwd(*args) == 6
    # the variant on the library's fixed scratch: same checks, then its own size limit, all before any HIP call
    na = lambda **kw: L.fa_bwd_noalloc(*[kw.get("ptr", p)] * 9, kw.get("B", 1), 1, kw.get("N", 16), kw.get("d", 128), 0.1, 0,
                                       kw.get("dtype", binding.FA_BF16), None)
    assert na(ptr=None) == 1 and na(d=96) == 4 and na(dtype=binding.FA_F32) == 4
    assert na(B=4, N=binding.FA_BWD_NOALLOC_MAX_ROWS // 4 + 1, d=64) == 8
    assert binding.status_string(8).startswith("problem exceeds")


def test_kernel_name_query_follows_the_launcher():
    # the benchmark attributes launches to kernels through this call; every request the forward accepts has a name
    name = binding.fa_fwd_kernel_name
    for dtype in (binding.FA_BF16, binding.FA_F16, binding.FA_FP8_E4M3):
        for d in (64, 128, 256):
            for N in (1, 512, 640, 641, 704, 705, 1280, 1281, 1408, 1409, 3072, 3073, 16384):
                for causal in (False, True):
                    n = name(dtype, N, d, causal)
                    assert n and n.startswith("fa_fwd_") and ("true" if causal else "false") in n
    assert name(binding.FA_F32, 256, 64, False) == "fa_fwd_f32_kernel<64, 32, false>"
    assert name(binding.FA_F32, 256, 128, False) is None and name(binding.FA_BF16, 256, 96, False) is None
    assert name(binding.FA_BF16, 0, 128, False) is None and name(9, 16, 128, False) is None
    # every kernel the benchmark holds a measured HBM-traffic figure for is one the launcher can still choose
    sweep = {name(dt, N, 128, c) for dt in (binding.FA_BF16, binding.FA_FP8_E4M3) for N in bench.SEQLENS
             for c in (False, True)}
    assert set(bench.MEASURED_TRAFFIC_BYTES_PER_LAUNCH) <= sweep


def test_mfma_probe_validates_and_counts_flops():
    L = binding.lib()
    # 512 workgroups x 8 waves x iters x 32 MFMAs of 2*32*32*16 (bf16) or 2*32*32*64 (e4m3) FLOPs
    assert L.fa_probe_mfma_flops(binding.FA_BF16, 10) == 512 * 8 * 10 * 32 * 2 * 32 * 32 * 16
    assert L.fa_probe_mfma_flops(binding.FA_FP8_E4M3, 10) == 512 * 8 * 10 * 32 * 2 * 32 * 32 * 64
    assert L.fa_probe_mfma_flops(binding.FA_F16, 10) == 0.0
    assert L.fa_probe_mfma(None, 1024, 16, binding.FA_BF16, 10, None) == 1
    assert L.fa_probe_mfma(16, 1024, 16, binding.FA_F16, 10, None) == 4
    assert L.fa_probe_mfma(16, 1000, 16, binding.FA_BF16, 10, None) == 2
    assert L.fa_probe_mfma(16, 1024, 16, binding.FA_BF16, 0, None) == 2
    assert L.fa_probe_mfma(8, 1024, 16, binding.FA_BF16, 10, None) == 5


def test_flop_accounting_matches_the_papers_ablation_table():
    import json
    g = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_values.json")))
    row = g["ablation_full_method"]
    fl = bench.attention_flops(row["batch"], row["nheads"], row["seqlen"], row["hdim"], row["causal"])
    assert fl / (row["time_ms"] * 1e-3) / 1e12 == pytest.approx(row["tflops"], abs=0.6)
    for name in ("ablation_no_pipelining", "ablation_no_warp_specialization"):
        assert fl / (g[name]["time_ms"] * 1e-3) / 1e12 == pytest.approx(g[name]["tflops"], abs=0.6)
    assert bench.attention_flops(1, 1, 8, 4, True) == 0.5 * bench.attention_flops(1, 1, 8, 4, False)
    assert bench.attention_flops(1, 1, 8, 4, False, backward=True) == g["flops_rule"]["bwd_over_fwd"] * bench.attention_flops(1, 1, 8, 4, False)
    # matmul FLOPs per exponential at head dim 128: 4*N^2*d / N^2 = 512
    e = g["exp_vs_matmul"]
    assert bench.attention_flops(1, 1, 64, e["hdim"], False) / (64 * 64) == e["matmul_flops_per_exp"]


def test_mfma_hazard_checker_finds_planted_early_access():
    """The build runs this checker over the backward kernels' assembly; here it is shown to see what
    it is for, on a listing written by hand."""
    from paper_2407_08608_amd import mfma_hazard_check as hz
    head = "_Z6kernelv:\n\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 v[16:31], v[0:3], a[0:3], 0\n\t;;#ASMEND\n"
    chain = "\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 v[16:31], v[4:7], a[4:7], v[16:31]\n\t;;#ASMEND\n"
    wait = "\ts_nop 12\n"
    read = "\tv_exp_f32_e32 v40, v17\n"
    assert hz.check(head + chain + wait + read) == []
    assert len(hz.check(head + chain + read)) == 1                       # VALU read right behind the MFMA
    assert len(hz.check(head + "\tv_mov_b32_e32 v50, v31\n" + chain + wait + read)) == 1   # a copy between two MFMAs
    assert len(hz.check(head + "\tds_read_b128 v[28:31], v60\n" + wait)) == 1              # overwritten too early
    assert len(hz.check(head + "\ts_nop 7\n\tv_mfma_f32_32x32x16_bf16 a[0:15], v[16:19], v[8:11], a[0:15]\n")) == 1
    # a reader at the head of a loop, reached only through the back-edge right behind the MFMA
    loop = "_Z6kernelv:\n.LBB0_1:\n" + read + "\ts_nop 12\n\t;;#ASMSTART\n\tv_mfma_f32_32x32x16_bf16 v[16:31], v[0:3], a[0:3], 0\n\t;;#ASMEND\n"
    assert len(hz.check(loop + "\ts_cbranch_scc1 .LBB0_1\n")) == 1
    assert hz.check(loop + wait + "\ts_cbranch_scc1 .LBB0_1\n") == []
    # a forward branch that skips the wait
    skip = head + "\ts_cbranch_vccz .LBB0_2\n" + wait + ".LBB0_2:\n" + read
    assert len(hz.check(skip)) == 1
    # an MFMA the compiler scheduled itself (no ASMSTART) is the compiler's business
    assert hz.check("_Z6kernelv:\n\tv_mfma_f32_32x32x16_bf16 v[16:31], v[0:3], v[4:7], 0\n" + read) == []


def test_bench_refuses_more_than_one_gpu_with_a_message():
    # the build measures one GPU; the benchmark says so instead of printing a line for several
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
