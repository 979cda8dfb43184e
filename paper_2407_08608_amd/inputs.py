"""Seeded synthetic inputs for tests and benchmarks.

This module holds none of the attention arithmetic: it only draws random tensors of the
shapes and distributions the paper benchmarks on (section 4.1 "Benchmark settings":
16k tokens in total, hidden size 2048; section 4.3: N(0,1) + N(0,100)*Bernoulli(0.001)
for the numerical-error study) and rounds them once to the storage dtype.  The same bits
are handed to the HIP library and (upcast exactly) to the CPU oracle.
"""
import numpy as np
import torch

_TORCH_DTYPES = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}


def _rng(seed, name):
    # independent stream per (seed, tensor name)
    tag = int.from_bytes(name.encode()[:8].ljust(8, b"\0"), "little")
    return np.random.Generator(np.random.PCG64([int(seed), tag]))


def normal_tensor(seed, name, shape, dtype="bf16"):
    """i.i.d. N(0,1) entries, rounded to `dtype`; a torch CPU tensor."""
    x = _rng(seed, name).standard_normal(size=shape, dtype=np.float32)
    return torch.from_numpy(x).to(_TORCH_DTYPES[dtype])


def heavy_tailed_tensor(seed, name, shape, dtype="bf16", p_outlier=0.001, outlier_std=10.0):
    """N(0,1) + N(0, outlier_std^2) * Bernoulli(p_outlier), the paper's error-study inputs."""
    g = _rng(seed, name)
    x = g.standard_normal(size=shape, dtype=np.float32)
    mask = g.random(size=shape, dtype=np.float32) < p_outlier
    x = x + mask * (outlier_std * g.standard_normal(size=shape, dtype=np.float32))
    return torch.from_numpy(x.astype(np.float32)).to(_TORCH_DTYPES[dtype])


def qkv(seed, B, H, N, d, dtype="bf16", heavy_tailed=False):
    make = heavy_tailed_tensor if heavy_tailed else normal_tensor
    return tuple(make(seed, n, (B, H, N, d), dtype) for n in ("q", "k", "v"))


def rising_maximum_qkv(seed, B, H, N, d, dtype="bf16", top_nats=80.0, beta=30.0):
    """An adversarial case for online softmax: with scale d^-1/2 the score of query i and key j is
    about top_nats * j / N plus N(0, ~3) noise, so every row's running maximum keeps rising from the
    first key block to the last.  q = g + beta u, k_j = h_j + (top_nats sqrt(d) j / (N beta)) u with
    g, h i.i.d. N(0,1) and u the unit vector along (1, ..., 1); v i.i.d. N(0,1)."""
    q, k, v = (normal_tensor(seed, n, (B, H, N, d), "f32") for n in ("q", "k", "v"))
    u = torch.full((d,), float(d) ** -0.5)
    ramp = torch.arange(N, dtype=torch.float32) * (top_nats * float(d) ** 0.5 / (N * beta))
    q = q + beta * u
    k = k + ramp[:, None] * u
    return tuple(t.to(_TORCH_DTYPES[dtype]) for t in (q, k, v))


def random_signs(seed, d):
    """The +-1 diagonal of the incoherent-processing matrix, int8 [d]."""
    s = _rng(seed, "signs").integers(0, 2, size=d) * 2 - 1
    return torch.from_numpy(s.astype(np.int8))


def sample_rows(seed, total_rows, n):
    """n distinct flat row indices in [0, total_rows), sorted, int64 numpy."""
    n = min(n, total_rows)
    return np.sort(_rng(seed, "rows").choice(total_rows, size=n, replace=False)).astype(np.int64)


def benchmark_shape(N, d, tokens=16384, hidden=2048):
    """(B, H) of the paper's sweep: batch = tokens / seqlen, heads = hidden / head_dim."""
    return tokens // N, hidden // d
