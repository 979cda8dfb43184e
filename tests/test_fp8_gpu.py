"""Parity of the FP8 pre-pass and FP8 forward (through the C ABI) against the oracles.

Pre-pass: codes are bytes and scales are fp32 values decided by fp32 arithmetic that the
oracle reproduces step by step, so both must match bit for bit.

Forward, against the model oracle (fp64 attention on the de-quantised tensors): the only
rounding the kernel adds is P~ -> e4m3 (at most 2^-4 of a normal P~, 2^-10 for a subnormal one)
and the bf16 store (2^-9 |O|).  Every output element is held to the bound that follows for its
own row (helpers.fp8_rounding_bound: 2^-4 of the P-weighted mean of |V^| over the keys the row
sees, plus the subnormal floor), on N(0,1) inputs and on the heavy-tailed inputs of the paper's
error study, where the lazily raised reference maximum and the accumulator rescale fire often.
L is computed in fp32 from exact fp8 products and must agree to 2e-3.

Forward, against the true fp64 attention on the original inputs (the paper's error study,
section 4.3): block quantisation + incoherent processing must beat per-tensor scaling on
heavy-tailed inputs.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import fp8_oracle as f8
from helpers import check_fp8_against_model_oracle, f64, gpu_rows, max_abs, rmse
from paper_2407_08608_amd import binding, inputs

pytestmark = pytest.mark.gpu


def _quant_gpu(x, signs, per_tensor=False):
    s = None if signs is None else signs.cuda()
    x8, sc = binding.fa_fp8_quant_hadamard(x.cuda(), s, 128, per_tensor)
    torch.cuda.synchronize()
    return x8.cpu().numpy(), sc.cpu().numpy()


@pytest.mark.parametrize("dtype", ["bf16", "f16", "f32"])
@pytest.mark.parametrize("use_signs", [False, True])
@pytest.mark.parametrize("d", [64, 128, 256])
def test_quant_codes_and_scales_bit_exact(d, use_signs, dtype):
    B, H, N = 2, 2, 300  # ragged last block
    x = inputs.heavy_tailed_tensor(20 + d, "x", (B, H, N, d), dtype)
    x[0, 1, 128:256] = 0  # an all-zero block
    signs = inputs.random_signs(21, d) if use_signs else None
    codes, scales = _quant_gpu(x, signs)
    c_ref, s_ref = f8.quantize(x.float().numpy(), None if signs is None else signs.numpy(), 128)
    np.testing.assert_array_equal(scales.view(np.uint32), s_ref.view(np.uint32))
    np.testing.assert_array_equal(codes, c_ref)


@pytest.mark.parametrize("use_signs", [False, True])
def test_quant_per_tensor_bit_exact(use_signs):
    B, H, N, d = 1, 3, 257, 128
    x = inputs.heavy_tailed_tensor(22, "x", (B, H, N, d), "bf16")
    signs = inputs.random_signs(23, d) if use_signs else None
    codes, scales = _quant_gpu(x, signs, per_tensor=True)
    c_ref, s_ref = f8.quantize(x.float().numpy(), None if signs is None else signs.numpy(), 128, per_tensor=True)
    np.testing.assert_array_equal(scales.view(np.uint32), s_ref.view(np.uint32))
    np.testing.assert_array_equal(codes, c_ref)


def test_quant_single_row_and_full_benchmark_block_count():
    x = inputs.normal_tensor(24, "x", (1, 1, 1, 64), "bf16")
    codes, scales = _quant_gpu(x, None)
    c_ref, s_ref = f8.quantize(x.float().numpy(), None, 128)
    np.testing.assert_array_equal(codes, c_ref)
    np.testing.assert_array_equal(scales, s_ref)
    # full-size tensor of the sweep (16k tokens x 2048): sampled blocks against the oracle
    B, H, N, d = 1, 16, 16384, 128
    x = inputs.heavy_tailed_tensor(25, "x", (B, H, N, d), "bf16")
    signs = inputs.random_signs(25, d)
    codes, scales = _quant_gpu(x, signs)
    assert scales.shape == (B, H, N // 128)
    for (h, t) in [(0, 0), (7, 63), (15, 127)]:
        blk = x[:, h:h + 1, t * 128:(t + 1) * 128].float().numpy()
        c_ref, s_ref = f8.quantize(blk, signs.numpy(), 128)
        np.testing.assert_array_equal(codes[:, h:h + 1, t * 128:(t + 1) * 128], c_ref)
        assert scales[0, h, t] == s_ref[0, 0, 0]


_PREPARED = {}  # the last problem prepared: consecutive cases differ in the mask only


def _prepare(seed, B, H, N, d, heavy, use_signs=True, per_tensor=False):
    """Quantise with the ORACLE (inputs to the kernel under test never come from the HIP path)."""
    key = (seed, B, H, N, d, heavy, use_signs, per_tensor)
    if key not in _PREPARED:
        _PREPARED.clear()
        _PREPARED[key] = _prepare_uncached(*key)
    return _PREPARED[key]


def _prepare_uncached(seed, B, H, N, d, heavy, use_signs, per_tensor):
    q, k, v = inputs.qkv(seed, B, H, N, d, "bf16", heavy_tailed=heavy)
    signs = inputs.random_signs(seed, d).numpy() if use_signs else None
    qc, qs = f8.quantize(q.float().numpy(), signs, 128, per_tensor)
    kc, ks = f8.quantize(k.float().numpy(), signs, 128, per_tensor)
    vc, vs = f8.quantize(v.float().numpy(), None, 128, per_tensor)
    return (q, k, v), (qc, kc, vc), (qs, ks, vs)


def _fwd_fp8_gpu(codes, scales, scale, causal):
    dev = [torch.from_numpy(c).cuda() for c in codes] + [torch.from_numpy(s).cuda() for s in scales]
    o, lse = binding.fa_fwd_fp8(*dev, scale, causal)
    torch.cuda.synchronize()
    return o, lse


@pytest.mark.parametrize("heavy", [False, True])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("d", [64, 128, 256])
@pytest.mark.parametrize("N", [1, 100, 256, 700, 1500])
def test_fp8_forward_matches_model_oracle(N, d, causal, heavy):
    # 1500 keys: past the length up to which d = 128 keeps its four-wave tile, with a ragged tail
    B, H = 2, 2
    # heavy: the inputs of the paper's error study (section 4.3), N(0,1) + N(0,100) Bernoulli(0.001)
    _, codes, scales = _prepare(30 + N + d, B, H, N, d, heavy=heavy)
    scale = d ** -0.5
    o, lse = _fwd_fp8_gpu(codes, scales, scale, causal)
    check_fp8_against_model_oracle(o, lse, codes, scales, scale, causal)


@pytest.mark.parametrize("heavy", [False, True])
def test_fp8_forward_d64_eight_wave_tile_ragged(heavy):
    # d = 64 without a mask switches to its 256-query tile only above 3072 keys
    B, H, N, d = 1, 2, 3300, 64
    _, codes, scales = _prepare(39, B, H, N, d, heavy=heavy)
    o, lse = _fwd_fp8_gpu(codes, scales, d ** -0.5, False)
    check_fp8_against_model_oracle(o, lse, codes, scales, d ** -0.5, False)


def test_fp8_forward_block_scales_really_differ_per_block():
    # make the blocks' scales very different so a wrong scale index cannot hide
    B, H, N, d = 1, 2, 512, 128
    q, k, v = inputs.qkv(40, B, H, N, d, "bf16")
    for t in range(4):
        k[:, :, t * 128:(t + 1) * 128] *= (0.25 * (t + 1))
        v[:, :, t * 128:(t + 1) * 128] *= (4.0 / (t + 1))
        q[:, :, t * 128:(t + 1) * 128] *= (0.5 + 0.5 * t)
    codes, scales = zip(*[f8.quantize(x.float().numpy(), None, 128) for x in (q, k, v)])
    assert scales[1][0, 0, 3] > 2 * scales[1][0, 0, 0]
    for causal in (False, True):
        o, lse = _fwd_fp8_gpu(codes, scales, d ** -0.5, causal)
        check_fp8_against_model_oracle(o, lse, codes, scales, d ** -0.5, causal)


@pytest.mark.parametrize("causal", [False, True])
def test_fp8_forward_v_scales_jump_up_and_down_by_large_factors(causal):
    # a V block's scale enters the kernel as an offset in the exponent of P~, and the reference maximum
    # is taken over the offset scores: make consecutive V blocks differ by factors far above and below
    # the lazy-raise threshold, with an all-zero block (scale 1 by convention) in the middle
    B, H, N, d = 1, 2, 1024, 128
    q, k, v = inputs.qkv(42, B, H, N, d, "bf16")
    for t, f in enumerate([1.0, 64.0, 0.02, 0.0, 3.0, 1.5, 0.001, 200.0]):
        v[:, :, t * 128:(t + 1) * 128] *= f
    codes, scales = zip(*[f8.quantize(x.float().numpy(), None, 128) for x in (q, k, v)])
    assert scales[2][0, 0, 3] == 1.0 and scales[2][0, 0, 1] > 30 * scales[2][0, 0, 0]
    o, lse = _fwd_fp8_gpu(codes, scales, d ** -0.5, causal)
    check_fp8_against_model_oracle(o, lse, codes, scales, d ** -0.5, causal)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(2300, 128), (2300, 256), (3300, 64), (600, 128)])
def test_fp8_row_maxima_that_rise_block_after_block(N, d, causal):
    # scores grow from ~0 at the first key to ~80 at the last, so the reference maximum (threshold 2 in
    # log2 units) rises in almost every key block; the d = 256 kernel applies the rescale one block
    # behind the scores
    q, k, v = inputs.rising_maximum_qkv(44, 1, 2, N, d, "bf16")
    codes, scales = zip(*[f8.quantize(x.float().numpy(), None, 128) for x in (q, k, v)])
    o, lse = _fwd_fp8_gpu(codes, scales, d ** -0.5, causal)
    check_fp8_against_model_oracle(o, lse, codes, scales, d ** -0.5, causal)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [333, 1500])
@pytest.mark.parametrize("d", [64, 128, 256])
def test_fp8_unit_scale_entry_point_matches_oracle(d, N, causal):
    """fa_fwd with dtype e4m3 takes the codes at unit scale: every kernel (the four-wave tiles at 333 keys, the
    eight-wave tiles at 1500) has an instantiation without block scales of its own."""
    B, H = 1, 2
    rng = np.random.default_rng(43 + d)
    qc, kc, vc = (f8.e4m3_encode(rng.standard_normal((B, H, N, d))) for _ in range(3))
    dev = [torch.from_numpy(c).cuda() for c in (qc, kc, vc)]
    o, lse = binding.fa_fwd(*dev, d ** -0.5, causal, dtype=binding.FA_FP8_E4M3)
    torch.cuda.synchronize()
    ones = np.ones((B, H, -(-N // 128)), dtype=np.float32)
    check_fp8_against_model_oracle(o, lse, (qc, kc, vc), (ones, ones, ones), d ** -0.5, causal)


def test_fp8_unit_scale_entry_point_and_constant_values():
    B, H, N, d = 1, 2, 200, 128
    rng = np.random.default_rng(41)
    qc, kc = (f8.e4m3_encode(rng.standard_normal((B, H, N, d))) for _ in range(2))
    row = f8.e4m3_encode(rng.standard_normal(d))
    vc = np.broadcast_to(row, (B, H, N, d)).copy()
    dev = [torch.from_numpy(c).cuda() for c in (qc, kc, vc)]
    o, lse = binding.fa_fwd(*dev, d ** -0.5, True, dtype=binding.FA_FP8_E4M3)
    torch.cuda.synchronize()
    o_ref, l_ref = oracle.attention_fwd(f8.e4m3_decode(qc), f8.e4m3_decode(kc), f8.e4m3_decode(vc), d ** -0.5, True)
    # all value rows equal: the output row is that row whatever P~ is (up to l vs sum of rounded P~)
    assert max_abs(f64(o), o_ref) <= 2.0 ** -4 * np.abs(f8.e4m3_decode(row)).max()
    assert max_abs(f64(lse), l_ref) <= 2e-3
    assert torch.equal(o[:, :, 0].float().cpu(), torch.from_numpy(f8.e4m3_decode(vc[:, :, 0])).float())


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("H,N,d,heavy", [(16, 16384, 128, False), (8, 16384, 256, False), (32, 16384, 64, False),
                                         (16, 4096, 128, False), (16, 16384, 128, True), (8, 16384, 256, True),
                                         (32, 16384, 64, True), (16, 4096, 128, True), (8, 4096, 256, True)])
def test_fp8_benchmark_shapes_sampled_rows(H, N, d, heavy, causal):
    """The shapes the benchmark times (section 4.1: 16k tokens in total, hidden size 2048), in the
    kernel and launch configuration it times, on N(0,1) inputs and on the heavy-tailed inputs of the
    error study (section 4.3); sampled output rows against the model oracle, element by element."""
    B = 16384 // N
    _, codes, scales = _prepare(70 + d, B, H, N, d, heavy=heavy)
    scale = d ** -0.5
    o, lse = _fwd_fp8_gpu(codes, scales, scale, causal)
    assert bool(torch.isfinite(o).all()) and bool(torch.isfinite(lse).all())
    rows = inputs.sample_rows(71 + d, B * H * N, 384)
    # the first and the last rows of a head, and both sides of a 128-row scale block boundary
    rows = np.unique(np.concatenate([rows, [0, 1, 127, 128, N - 1, N, B * H * N - 1]])).astype(np.int64)
    got, o_ref = check_fp8_against_model_oracle(o, lse, codes, scales, scale, causal, rows=rows)
    # long rows average the P~ rounding down; causal rows are as short as one key
    if not heavy:
        assert rmse(got, o_ref) <= (8e-3 if causal else 2e-3)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(4096, 128), (4096, 256), (16384, 128), (16384, 256), (4096, 64)])
def test_fp8_error_ordering_on_heavy_tailed_inputs_full_gpu_path(N, d, causal):
    """Section 4.3 / Table 3: quantisation pre-pass and forward both on the GPU, error against
    fp64 attention on the original inputs, at points of the sweep (16k tokens, hidden size 2048);
    sampled rows."""
    B, H = inputs.benchmark_shape(N, d)
    q, k, v = inputs.qkv(50, B, H, N, d, "bf16", heavy_tailed=True)
    signs = inputs.random_signs(50, d).cuda()
    qg, kg, vg = q.cuda(), k.cuda(), v.cuda()
    scale = d ** -0.5
    rows = inputs.sample_rows(51, B * H * N, 512)
    o_ref, _ = oracle.attention_fwd_rows(f64(q), f64(k), f64(v), rows, scale, causal)

    def run(sg, per_tensor):
        q8, qs = binding.fa_fp8_quant_hadamard(qg, sg, 128, per_tensor)
        k8, ks = binding.fa_fp8_quant_hadamard(kg, sg, 128, per_tensor)
        v8, vs = binding.fa_fp8_quant_hadamard(vg, None, 128, per_tensor)
        o, _ = binding.fa_fwd_fp8(q8, k8, v8, qs, ks, vs, scale, causal)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(o).all())
        return rmse(gpu_rows(o, rows), o_ref)

    full = run(signs, False)
    baseline = run(None, True)
    no_block = run(signs, True)
    no_incoh = run(None, False)
    print(f"fp8 rmse N={N} d={d} causal={causal}: full={full:.3e} baseline={baseline:.3e} "
          f"no_block_quant={no_block:.3e} no_incoherent={no_incoh:.3e}")
    assert full < baseline
    assert full < 5e-2
