"""Parity of the HIP backward (through the C ABI) against the fp64 oracle.

The GPU backward is fed what training would feed it: the bf16 O and fp32 L written by the GPU
forward, and bf16 dO.  The oracle differentiates the exact fp64 attention of the same stored
Q, K, V.  The paper states no tolerance for gradients; the bound used here (relative RMSE
<= 1e-2 per tensor, max-abs <= 5e-2 of the reference's largest magnitude) follows from bf16
rounding (2^-9 relative) of P, dS and O entering 128..16k-term fp32 sums.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import f64, gpu_rows, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu

REL_RMSE, REL_MAXABS = 1e-2, 5e-2


def _gpu_bwd(q, k, v, dout, scale, causal):
    qg, kg, vg, dog = (t.cuda() for t in (q, k, v, dout))
    o, lse = binding.fa_fwd(qg, kg, vg, scale, causal)
    dq, dk, dv = binding.fa_bwd(qg, kg, vg, o, lse, dog, scale, causal)
    torch.cuda.synchronize()
    return dq, dk, dv


def _compare(got, ref, name):
    g = f64(got)
    assert np.isfinite(g).all(), name
    # absolute floors cover references that are exactly zero (e.g. dQ, dK with a single key)
    err, ma = rmse(g, ref), max_abs(g, ref)
    ref_rms = float(np.sqrt(np.mean(ref * ref)))
    assert err <= REL_RMSE * ref_rms + 1e-5 and ma <= REL_MAXABS * np.abs(ref).max() + 1e-4, \
        (name, err, ref_rms, ma, float(np.abs(ref).max()))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("N", [1, 40, 64, 129, 257, 600])
def test_bwd_small_and_ragged(N, d, causal, dtype):
    B, H = 2, 2
    q, k, v = inputs.qkv(60 + N, B, H, N, d, dtype)
    dout = inputs.normal_tensor(61 + N, "do", (B, H, N, d), dtype)
    scale = d ** -0.5
    dq, dk, dv = _gpu_bwd(q, k, v, dout, scale, causal)
    ref = oracle.attention_bwd(f64(q), f64(k), f64(v), f64(dout), scale, causal)
    _compare(dq, ref["dq"], "dq")
    _compare(dk, ref["dk"], "dk")
    _compare(dv, ref["dv"], "dv")


def test_bwd_constant_values_give_zero_query_and_key_gradients():
    B, H, N, d = 1, 2, 256, 128
    q, k, v = inputs.qkv(70, B, H, N, d, "bf16")
    v = v[:, :, :1].expand(B, H, N, d).contiguous()
    dout = inputs.normal_tensor(71, "do", (B, H, N, d), "bf16")
    dq, dk, dv = _gpu_bwd(q, k, v, dout, d ** -0.5, False)
    # dP - D vanishes up to the bf16 rounding of O: gradients are tiny compared with |dO| ~ 1
    assert float(dq.float().abs().max()) <= 5e-2 and float(dk.float().abs().max()) <= 5e-2
    # columns of dV sum to the column sums of dO (P is row-stochastic)
    np.testing.assert_allclose(f64(dv).sum(axis=2), f64(dout).sum(axis=2), rtol=2e-2, atol=0.3)


def test_bwd_is_repeatable_and_workspace_checked():
    B, H, N, d = 1, 2, 300, 128
    q, k, v = inputs.qkv(72, B, H, N, d, "bf16")
    dout = inputs.normal_tensor(73, "do", (B, H, N, d), "bf16")
    a = _gpu_bwd(q, k, v, dout, d ** -0.5, True)
    b = _gpu_bwd(q, k, v, dout, d ** -0.5, True)
    assert all(torch.equal(x, y) for x, y in zip(a, b))  # no atomics: fixed summation order
    need = binding.fa_bwd_workspace_bytes(B, H, N, d)
    assert need >= B * H * N * 4  # D = rowsum(dO o O)
    small = torch.empty(need - 16, device="cuda", dtype=torch.uint8)
    with pytest.raises(binding.FaError) as e:
        qg = q.cuda()
        binding.fa_bwd(qg, qg, qg, qg, torch.empty(B, H, N, device="cuda"), qg, 0.1, False, workspace=small)
    assert e.value.status == 6


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(1024, 128), (4096, 128), (16384, 128), (4096, 64), (16384, 64), (4096, 256),
                                 (16384, 256)])
def test_bwd_benchmark_shapes_sampled_heads(N, d, causal):
    # 16k tokens, hidden size 2048 (16 heads of dim 128 or 32 of dim 64); the oracle differentiates
    # whole (batch, head) slices
    B, H = inputs.benchmark_shape(N, d)
    q, k, v = inputs.qkv(80, B, H, N, d, "bf16")
    dout = inputs.normal_tensor(81, "do", (B, H, N, d), "bf16")
    scale = d ** -0.5
    dq, dk, dv = _gpu_bwd(q, k, v, dout, scale, causal)
    assert all(bool(torch.isfinite(t).all()) for t in (dq, dk, dv))
    picks = [(0, 0), (B - 1, H - 1)] if N <= 4096 else [(0, 5)]
    for (b, h) in picks:
        sl = (slice(b, b + 1), slice(h, h + 1))
        ref = oracle.attention_bwd(f64(q[sl]), f64(k[sl]), f64(v[sl]), f64(dout[sl]), scale, causal)
        _compare(dq[sl], ref["dq"], f"dq[{b},{h}]")
        _compare(dk[sl], ref["dk"], f"dk[{b},{h}]")
        _compare(dv[sl], ref["dv"], f"dv[{b},{h}]")


@pytest.mark.parametrize("causal", [False, True])
def test_bwd_long_ragged_sequence_sampled(causal):
    """Half a million keys, not a multiple of any tile: far longer than the oracle can differentiate
    whole, so it checks dQ on sampled query rows and, under the causal mask, dK and dV of the last
    205 keys (the ragged last key block and the full one before it), which only the last queries
    reach.  Those tail gradients are tiny (P ~ 1/N), so they are compared relative to their own size."""
    B, H, N, d = 1, 2, 524288 + 77, 128
    q, k, v = inputs.qkv(90, B, H, N, d, "bf16")
    dout = inputs.normal_tensor(91, "do", (B, H, N, d), "bf16")
    scale = d ** -0.5
    dq, dk, dv = _gpu_bwd(q, k, v, dout, scale, causal)
    assert all(bool(torch.isfinite(t).all()) for t in (dq, dk, dv))
    q64, k64, v64, do64 = f64(q), f64(k), f64(v), f64(dout)
    rows = np.unique(np.concatenate([inputs.sample_rows(92, B * H * N, 60), [1, N - 1, N, 2 * N - 1]])).astype(np.int64)
    ref = oracle.attention_bwd_dq_rows(q64, k64, v64, do64, rows, scale, causal)
    got = gpu_rows(dq, rows)
    ref_rms = float(np.sqrt(np.mean(ref * ref)))
    assert rmse(got, ref) <= REL_RMSE * ref_rms and max_abs(got, ref) <= REL_MAXABS * np.abs(ref).max(), \
        (rmse(got, ref), ref_rms, max_abs(got, ref))
    if causal:
        j0 = N - 77 - 128
        for h in range(H):
            dk_ref, dv_ref = oracle.attention_bwd_dkdv_keys(q64[0, h], k64[0, h], v64[0, h], do64[0, h], j0, N,
                                                            scale, True)
            for name, g, r in (("dk", dk, dk_ref), ("dv", dv, dv_ref)):
                g = f64(g[0, h, j0:])
                r_rms = float(np.sqrt(np.mean(r * r)))
                assert rmse(g, r) <= REL_RMSE * r_rms and max_abs(g, r) <= REL_MAXABS * np.abs(r).max(), \
                    (name, h, rmse(g, r), r_rms, max_abs(g, r))
