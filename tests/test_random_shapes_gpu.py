"""Seeded random shapes through every attention entry point against the fp64 oracle.

The fixed-shape tests pick lengths by hand; here lengths are drawn around every boundary where the
launcher changes kernels or a tile becomes ragged (multiples of 32, 64, 128, 256 plus or minus a
few rows; the lengths 640, 704, 1280, 1408 and 3072 at which the forward switches tiles), with the
batch, head and group counts drawn as well.  Tolerances are those of the fixed-shape tests.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import fp8_oracle as f8
from helpers import check_fp8_against_model_oracle, f64, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu

O_MAXABS, O_RMSE, L_MAXABS = 2e-2, 3e-3, 2e-3
REL_RMSE, REL_MAXABS = 1e-2, 5e-2
EDGES = (32, 64, 128, 256, 512, 640, 704, 768, 1024, 1280, 1408, 1536)


def _draw_shapes(seed, count, n_max):
    rng = np.random.default_rng(seed)
    shapes = []
    for _ in range(count):
        edge = int(rng.choice([e for e in EDGES if e <= n_max]))
        N = max(1, edge + int(rng.integers(-3, 4)))
        if rng.random() < 0.3:
            N = int(rng.integers(1, n_max + 1))
        d = int(rng.choice([64, 128, 256]))
        H_kv = int(rng.choice([1, 2, 3]))
        group = int(rng.choice([1, 1, 2, 4]))
        B = int(rng.choice([1, 2, 3]))
        shapes.append((B, H_kv * group, H_kv, N, d, bool(rng.integers(0, 2)), str(rng.choice(["bf16", "f16"]))))
    return shapes


@pytest.mark.parametrize("B,H,H_kv,N,d,causal,dtype", _draw_shapes(20240711, 36, 1540))
def test_forward_random_shape(B, H, H_kv, N, d, causal, dtype):
    q = inputs.normal_tensor(7 * N + d, "q", (B, H, N, d), dtype)
    k = inputs.normal_tensor(7 * N + d, "k", (B, H_kv, N, d), dtype)
    v = inputs.normal_tensor(7 * N + d, "v", (B, H_kv, N, d), dtype)
    scale = d ** -0.5
    o, lse = binding.fa_fwd_gqa(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    torch.cuda.synchronize()
    o_ref, l_ref = oracle.attention_fwd_gqa(f64(q), f64(k), f64(v), scale, causal)
    assert np.isfinite(f64(o)).all() and np.isfinite(f64(lse)).all()
    e_o, r_o, e_l = max_abs(f64(o), o_ref), rmse(f64(o), o_ref), max_abs(f64(lse), l_ref)
    assert e_o <= O_MAXABS and r_o <= O_RMSE and e_l <= L_MAXABS, (e_o, r_o, e_l)


@pytest.mark.parametrize("B,H,H_kv,N,d,causal,dtype", _draw_shapes(20240712, 24, 800))
def test_backward_random_shape(B, H, H_kv, N, d, causal, dtype):
    q = inputs.normal_tensor(9 * N + d, "q", (B, H, N, d), dtype)
    k = inputs.normal_tensor(9 * N + d, "k", (B, H_kv, N, d), dtype)
    v = inputs.normal_tensor(9 * N + d, "v", (B, H_kv, N, d), dtype)
    dout = inputs.normal_tensor(9 * N + d, "do", (B, H, N, d), dtype)
    scale = d ** -0.5
    qg, kg, vg, dog = (t.cuda() for t in (q, k, v, dout))
    o, lse = binding.fa_fwd_gqa(qg, kg, vg, scale, causal)
    dq, dk, dv = binding.fa_bwd_gqa(qg, kg, vg, o, lse, dog, scale, causal)
    torch.cuda.synchronize()
    ref = oracle.attention_bwd_gqa(f64(q), f64(k), f64(v), f64(dout), scale, causal)
    for name, got in (("dq", dq), ("dk", dk), ("dv", dv)):
        g, r = f64(got), ref[name]
        assert np.isfinite(g).all(), name
        ref_rms = float(np.sqrt(np.mean(r * r)))
        assert rmse(g, r) <= REL_RMSE * ref_rms + 1e-5 and max_abs(g, r) <= REL_MAXABS * np.abs(r).max() + 1e-4, name


@pytest.mark.parametrize("B,H,H_kv,N,d,causal,dtype", _draw_shapes(20240713, 24, 1540))
def test_fp8_forward_random_shape(B, H, H_kv, N, d, causal, dtype):
    # quantised by the oracle; the reference is fp64 attention on the dequantised tensors
    # every other case on the heavy-tailed inputs of the paper's error study (section 4.3)
    make = inputs.heavy_tailed_tensor if (N + B + H) % 2 else inputs.normal_tensor
    q = make(11 * N + d, "q", (B, H, N, d), "bf16")
    k = make(11 * N + d, "k", (B, H_kv, N, d), "bf16")
    v = make(11 * N + d, "v", (B, H_kv, N, d), "bf16")
    signs = inputs.random_signs(N + d, d).numpy()
    (qc, qs), (kc, ks), (vc, vs) = (f8.quantize(x.float().numpy(), s, 128) for x, s in ((q, signs), (k, signs), (v, None)))
    scale = d ** -0.5
    dev = [torch.from_numpy(a).cuda() for a in (qc, kc, vc, qs, ks, vs)]
    o, lse = binding.fa_fwd_fp8_gqa(*dev, scale, causal)
    torch.cuda.synchronize()
    check_fp8_against_model_oracle(o, lse, (qc, kc, vc), (qs, ks, vs), scale, causal, kv_heads=H_kv)
