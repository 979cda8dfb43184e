"""Build libfa_mi355.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libfa_mi355.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # hipcc -O3 otherwise emits packed-fp32 VALU ops for plain float code
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# "#pragma unroll" silently leaves a loop rolled when its unrolled size passes a threshold; the
# backward kernels index register arrays by the loop variable and must be unrolled whatever their size.
EXTRA_FLAGS = {"fa_bwd.hip": ["-mllvm", "-pragma-unroll-threshold=1000000"]}


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    extra = EXTRA_FLAGS.get(os.path.basename(src), [])
    subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], check=True)
    return obj


# Sources with MFMAs written as inline assembly: their device assembly is generated once more as
# text and checked for instructions that touch an MFMA result too early (mfma_hazard_check.py).
HAZARD_CHECKED = ["fa_bwd.hip", "fa_fwd.hip"]


def _check_hazards(name):
    from . import mfma_hazard_check
    src, listing = os.path.join(CSRC, name), os.path.join(OBJ, name + ".s")
    subprocess.run([HIPCC, *FLAGS, *EXTRA_FLAGS.get(name, []), "-S", "--cuda-device-only", src, "-o", listing],
                   check=True, stderr=subprocess.DEVNULL)
    problems = mfma_hazard_check.check(open(listing).read())
    if problems:
        lines = "\n".join(f"  {f} +{ln}: {text} ({waited} wait states)" for f, ln, text, waited in problems[:20])
        raise RuntimeError(f"{name}: {len(problems)} accesses to the result of an inline-assembly MFMA come too early:\n{lines}")
    return name


def build(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    srcs = sorted(glob.glob(os.path.join(CSRC, "*.hip")))
    with ThreadPoolExecutor(max_workers=min(8, len(srcs) + len(HAZARD_CHECKED))) as ex:
        checks = [ex.submit(_check_hazards, n) for n in HAZARD_CHECKED]
        objs = list(ex.map(_compile, srcs))
        for c in checks:
            c.result()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
