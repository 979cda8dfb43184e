"""Parity of the multi-query / grouped-query entry points (section 3.1, "Attention variants")
against the fp64 oracle: K and V carry H_kv heads, query head h reads head h // (H / H_kv), and
dK, dV are sums over each group's query heads.  Tolerances are those of the ordinary forward and
backward tests (a group of G heads adds G times as many terms to dK and dV, all rounded the same way).
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import fp8_oracle as f8
from helpers import f64, gpu_rows, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu

O_MAXABS, O_RMSE, L_MAXABS = 2e-2, 3e-3, 2e-3
REL_RMSE, REL_MAXABS = 1e-2, 5e-2


def _tensors(seed, B, H, H_kv, N, d, dtype):
    q = inputs.normal_tensor(seed, "q", (B, H, N, d), dtype)
    k = inputs.normal_tensor(seed, "k", (B, H_kv, N, d), dtype)
    v = inputs.normal_tensor(seed, "v", (B, H_kv, N, d), dtype)
    return q, k, v


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,H_kv", [(4, 4), (4, 2), (6, 2), (3, 1)])
@pytest.mark.parametrize("N,d", [(129, 64), (300, 128), (1100, 128), (200, 256)])
def test_gqa_forward_16bit(N, d, H, H_kv, causal, dtype):
    # N = 1100 at d = 128 runs the ping-pong kernel when non-causal, the others the lock-step tiles
    B = 2
    q, k, v = _tensors(100 + N + H, B, H, H_kv, N, d, dtype)
    scale = d ** -0.5
    o, lse = binding.fa_fwd_gqa(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    torch.cuda.synchronize()
    o_ref, l_ref = oracle.attention_fwd_gqa(f64(q), f64(k), f64(v), scale, causal)
    e_o, r_o, e_l = max_abs(f64(o), o_ref), rmse(f64(o), o_ref), max_abs(f64(lse), l_ref)
    assert e_o <= O_MAXABS and r_o <= O_RMSE and e_l <= L_MAXABS, (e_o, r_o, e_l)


def test_gqa_forward_causal_pingpong_and_fp32():
    B, H, H_kv, N, d = 1, 4, 2, 2300, 128
    q, k, v = _tensors(110, B, H, H_kv, N, d, "bf16")
    o, lse = binding.fa_fwd_gqa(q.cuda(), k.cuda(), v.cuda(), d ** -0.5, True)
    o_ref, l_ref = oracle.attention_fwd_gqa(f64(q), f64(k), f64(v), d ** -0.5, True)
    assert max_abs(f64(o), o_ref) <= O_MAXABS and rmse(f64(o), o_ref) <= O_RMSE and max_abs(f64(lse), l_ref) <= L_MAXABS
    q, k, v = _tensors(111, 2, 6, 3, 130, 64, "f32")
    for causal in (False, True):
        o, lse = binding.fa_fwd_gqa(q.cuda(), k.cuda(), v.cuda(), 0.125, causal)
        o_ref, l_ref = oracle.attention_fwd_gqa(f64(q), f64(k), f64(v), 0.125, causal)
        assert max_abs(f64(o), o_ref) <= 2e-5 and max_abs(f64(lse), l_ref) <= 2e-5


def test_gqa_equals_ordinary_entry_point_on_repeated_heads_bitwise():
    # the grouped kernel reads the same bits an ordinary launch reads from K, V repeated per group
    B, H, H_kv, N, d = 2, 8, 2, 1300, 128
    q, k, v = (t.cuda() for t in _tensors(112, B, H, H_kv, N, d, "bf16"))
    for causal in (False, True):
        o1, l1 = binding.fa_fwd_gqa(q, k, v, d ** -0.5, causal)
        kr = k.repeat_interleave(H // H_kv, dim=1).contiguous()
        vr = v.repeat_interleave(H // H_kv, dim=1).contiguous()
        o2, l2 = binding.fa_fwd(q, kr, vr, d ** -0.5, causal)
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,H_kv", [(4, 2), (4, 1)])
@pytest.mark.parametrize("d", [64, 128, 256])
def test_gqa_forward_fp8_block_scaled(d, H, H_kv, causal):
    B, N = 2, 300
    q, k, v = _tensors(120 + d + H_kv, B, H, H_kv, N, d, "bf16")
    signs = inputs.random_signs(121, d).numpy()
    qc, qs = f8.quantize(q.float().numpy(), signs, 128)
    kc, ks = f8.quantize(k.float().numpy(), signs, 128)
    vc, vs = f8.quantize(v.float().numpy(), None, 128)
    # distinct scales per key/value head so that a wrong scale row cannot hide
    ks = ks * (1.0 + np.arange(H_kv, dtype=np.float32))[None, :, None]
    vs = vs * (2.0 - 0.5 * np.arange(H_kv, dtype=np.float32))[None, :, None]
    dev = [torch.from_numpy(np.ascontiguousarray(x)).cuda() for x in (qc, kc, vc, qs, ks, vs)]
    scale = d ** -0.5
    o, lse = binding.fa_fwd_fp8_gqa(*dev, scale, causal)
    torch.cuda.synchronize()
    deq = [f8.dequantize(c, s, 128) for c, s in ((qc, qs), (kc, ks), (vc, vs))]
    o_ref, l_ref = oracle.attention_fwd_gqa(*deq, scale, causal)
    assert max_abs(f64(o), o_ref) <= 2.0 ** -4 * np.abs(deq[2]).max() * 1.05 + 2.0 ** -7
    assert max_abs(f64(lse), l_ref) <= 2e-3


def _compare(got, ref, name):
    g = f64(got)
    assert np.isfinite(g).all(), name
    err, ma = rmse(g, ref), max_abs(g, ref)
    ref_rms = float(np.sqrt(np.mean(ref * ref)))
    assert err <= REL_RMSE * ref_rms + 1e-5 and ma <= REL_MAXABS * np.abs(ref).max() + 1e-4, \
        (name, err, ref_rms, ma, float(np.abs(ref).max()))


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,H_kv", [(4, 4), (4, 2), (6, 2), (3, 1)])
@pytest.mark.parametrize("N", [1, 129, 333])
def test_gqa_backward(N, H, H_kv, causal, dtype):
    B, d = 2, 128
    q, k, v = _tensors(130 + N + H, B, H, H_kv, N, d, dtype)
    dout = inputs.normal_tensor(131 + N, "do", (B, H, N, d), dtype)
    scale = d ** -0.5
    qg, kg, vg, dog = (t.cuda() for t in (q, k, v, dout))
    o, lse = binding.fa_fwd_gqa(qg, kg, vg, scale, causal)
    dq, dk, dv = binding.fa_bwd_gqa(qg, kg, vg, o, lse, dog, scale, causal)
    torch.cuda.synchronize()
    assert dk.shape == k.shape and dv.shape == v.shape
    ref = oracle.attention_bwd_gqa(f64(q), f64(k), f64(v), f64(dout), scale, causal)
    _compare(dq, ref["dq"], "dq")
    _compare(dk, ref["dk"], "dk")
    _compare(dv, ref["dv"], "dv")


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,H_kv", [(4, 2), (3, 1)])
@pytest.mark.parametrize("d", [64, 256])
def test_gqa_backward_other_head_dims(d, H, H_kv, causal):
    B, N = 2, 333
    q, k, v = _tensors(160 + d + H, B, H, H_kv, N, d, "bf16")
    dout = inputs.normal_tensor(161 + d, "do", (B, H, N, d), "bf16")
    scale = d ** -0.5
    qg, kg, vg, dog = (t.cuda() for t in (q, k, v, dout))
    o, lse = binding.fa_fwd_gqa(qg, kg, vg, scale, causal)
    dq, dk, dv = binding.fa_bwd_gqa(qg, kg, vg, o, lse, dog, scale, causal)
    torch.cuda.synchronize()
    ref = oracle.attention_bwd_gqa(f64(q), f64(k), f64(v), f64(dout), scale, causal)
    _compare(dq, ref["dq"], "dq")
    _compare(dk, ref["dk"], "dk")
    _compare(dv, ref["dv"], "dv")


def test_gqa_backward_is_repeatable_and_rejects_bad_groups():
    B, H, H_kv, N, d = 1, 4, 2, 700, 128
    q, k, v = (t.cuda() for t in _tensors(140, B, H, H_kv, N, d, "bf16"))
    dout = inputs.normal_tensor(141, "do", (B, H, N, d), "bf16").cuda()
    o, lse = binding.fa_fwd_gqa(q, k, v, d ** -0.5, True)
    a = binding.fa_bwd_gqa(q, k, v, o, lse, dout, d ** -0.5, True)
    b = binding.fa_bwd_gqa(q, k, v, o, lse, dout, d ** -0.5, True)
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    L = binding.lib()
    p = q.data_ptr()
    assert L.fa_fwd_gqa(p, p, p, p, lse.data_ptr(), B, H, 3, N, d, 0.1, 0, binding.FA_BF16, None) == 2
    assert L.fa_fwd_gqa(p, p, p, p, lse.data_ptr(), B, H, 0, N, d, 0.1, 0, binding.FA_BF16, None) == 2
    assert L.fa_bwd_gqa(p, p, p, p, lse.data_ptr(), p, p, p, p, p, 1 << 20, B, H, 3, N, d, 0.1, 0,
                        binding.FA_BF16, None) == 2


@pytest.mark.parametrize("causal", [False, True])
def test_gqa_benchmark_shape_sampled_rows(causal):
    # the sweep's 16k-token shape at seqlen 4096 with 16 query heads on 4 key/value heads
    N, d, H, H_kv = 4096, 128, 16, 4
    B = 16384 // N
    q, k, v = _tensors(150, B, H, H_kv, N, d, "bf16")
    scale = d ** -0.5
    o, lse = binding.fa_fwd_gqa(q.cuda(), k.cuda(), v.cuda(), scale, causal)
    rows = inputs.sample_rows(151, B * H * N, 256)
    kr = np.repeat(f64(k), H // H_kv, axis=1)
    vr = np.repeat(f64(v), H // H_kv, axis=1)
    o_ref, l_ref = oracle.attention_fwd_rows(f64(q), kr, vr, rows, scale, causal)
    assert max_abs(gpu_rows(o, rows), o_ref) <= O_MAXABS and rmse(gpu_rows(o, rows), o_ref) <= O_RMSE
    assert max_abs(gpu_rows(lse, rows), l_ref) <= L_MAXABS
