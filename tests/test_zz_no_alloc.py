"""fa_bwd_noalloc (the backward on the library's fixed device scratch, for callers that cannot
allocate) against fa_bwd: same kernels, so the results must be equal bit for bit; and against the
fp64 oracle to the backward's tolerance.  Two calls in a row, the second on a smaller problem, so
that whatever the first left in the shared scratch is there when the second runs."""
import numpy as np
import pytest
import torch

import oracle
from helpers import f64, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu

REL_RMSE, REL_MAXABS = 1e-2, 5e-2


def _case(seed, B, H, N, d, causal, dtype="bf16"):
    q, k, v = inputs.qkv(seed, B, H, N, d, dtype)
    dout = inputs.normal_tensor(seed + 1, "do", (B, H, N, d), dtype)
    qg, kg, vg, dog = (t.cuda() for t in (q, k, v, dout))
    scale = d ** -0.5
    o, lse = binding.fa_fwd(qg, kg, vg, scale, causal)
    want = binding.fa_bwd(qg, kg, vg, o, lse, dog, scale, causal)
    outs = [torch.full_like(qg, float("nan")) for _ in range(3)]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = binding.fa_bwd_noalloc(qg, kg, vg, o, lse, dog, scale, causal, *outs)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name, g, w in zip(("dq", "dk", "dv"), got, want):
        assert torch.equal(g, w), name
    ref = oracle.attention_bwd(f64(q), f64(k), f64(v), f64(dout), scale, causal)
    for name, g in zip(("dq", "dk", "dv"), got):
        g, r = f64(g), ref[name]
        ref_rms = float(np.sqrt(np.mean(r * r)))
        assert np.isfinite(g).all()
        assert rmse(g, r) <= REL_RMSE * ref_rms + 1e-5 and max_abs(g, r) <= REL_MAXABS * np.abs(r).max() + 1e-4, name


@pytest.mark.parametrize("d,causal", [(128, True), (64, False), (256, True)])
def test_noalloc_backward_two_calls_second_smaller(d, causal):
    _case(300 + d, 2, 3, 700, d, causal)
    _case(310 + d, 1, 2, 129, d, causal)


def test_noalloc_backward_rejects_what_exceeds_its_scratch():
    B, H, N, d = 1, 2, binding.FA_BWD_NOALLOC_MAX_ROWS // 2 + 1, 64
    x = torch.empty((B, H, N, d), device="cuda", dtype=torch.bfloat16)
    lse = torch.empty((B, H, N), device="cuda", dtype=torch.float32)
    with pytest.raises(binding.FaError) as e:
        binding.fa_bwd_noalloc(x, x, x, x, lse, x, 0.125, False, x, x, x)
    assert e.value.status == 8
    # exactly at the limit is accepted
    N = binding.FA_BWD_NOALLOC_MAX_ROWS // 2
    x = x[:, :, :N].contiguous().normal_()
    lse = lse[:, :, :N].contiguous().zero_()
    outs = [torch.empty_like(x) for _ in range(3)]
    binding.fa_bwd_noalloc(x, x, x, x, lse, x, 0.125, True, *outs)
    torch.cuda.synchronize()
