"""Shared test helpers: exact upcasts for the oracle and error metrics."""
import numpy as np
import torch

import oracle as _oracle
from oracle import fp8_oracle as _f8


def f64(t):
    """Stored bits of a torch tensor, upcast exactly to a float64 numpy array."""
    return t.detach().cpu().double().numpy()


def max_abs(a, b):
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if np.size(a) else 0.0


def rmse(a, b):
    d = np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)
    return float(np.sqrt(np.mean(d * d))) if d.size else 0.0


def rel_rmse(a, ref):
    ref = np.asarray(ref, dtype=np.float64)
    return rmse(a, ref) / max(float(np.sqrt(np.mean(ref * ref))), 1e-300)


def gpu_rows(t, rows):
    """Rows `rows` (flat over B*H*N) of a [B,H,N,d] or [B,H,N] device tensor, as float64 numpy."""
    idx = torch.from_numpy(rows).to(t.device)
    flat = t.reshape(-1, t.shape[-1]) if t.dim() == 4 else t.reshape(-1)
    return flat.index_select(0, idx).double().cpu().numpy()


def fp8_rounding_bound(q_hat, k_hat, v_codes, v_scales, rows, alpha, causal, block_rows=128):
    """Per-element bound on what rounding P~ to e4m3 can do to the FP8 forward's output rows.

    The kernel computes O = sum_k round(P~_k) v8_k / sum_k (P~_k / s_V(k)) with v8 the decoded V codes and
    P~_k proportional to p_k s_V(k), normalised so that its row maximum is at least 2^6 (the bias; a lazily
    raised reference only makes it larger).  Rounding to e4m3 changes a normal P~ by at most 2^-4 of itself
    and a subnormal one by at most 2^-10, so with the smallest normalisation the output moves by at most
        sum_k max(2^-4 P~_k, 2^-10) |v8_kc| / sum_k (P~_k / s_V(k)).
    The first alternative alone is 2^-4 times the P-weighted mean of |V^|.  q_hat, k_hat: dequantised
    [B,H,N,d] float64; v_codes: decoded V codes (no scale) [B,H,N,d]; v_scales: [B,H,blocks]; rows: flat
    indices into B*H*N.  Returns [len(rows), d].
    """
    B, H, N, d = q_hat.shape
    sv = np.repeat(np.asarray(v_scales, dtype=np.float64), block_rows, axis=2)[:, :, :N]
    out = np.empty((len(rows), d))
    rows = np.asarray(rows, dtype=np.int64)
    heads = rows // N
    for bh in np.unique(heads):
        sel = np.nonzero(heads == bh)[0]
        b, h = divmod(int(bh), H)
        i = rows[sel] % N
        s = alpha * (q_hat[b, h, i] @ k_hat[b, h].T)  # [n, N]
        if causal:
            s = np.where(np.arange(N)[None, :] <= i[:, None], s, -np.inf)
        logw = s + np.log(sv[b, h])[None, :]
        pt = 64.0 * np.exp(logw - logw.max(axis=1, keepdims=True))
        num = np.maximum(2.0 ** -4 * pt, np.where(np.isfinite(s), 2.0 ** -10, 0.0)) @ np.abs(v_codes[b, h])
        den = (pt / sv[b, h][None, :]).sum(axis=1, keepdims=True)
        out[sel] = num / den
    return out


def check_fp8_against_model_oracle(o, lse, codes, scales, scale, causal, rows=None, kv_heads=None):
    """Element by element: O within the P~-rounding bound of its own row, L within 2e-3."""
    if kv_heads is not None:  # grouped-query: repeat K, V per group for the oracle
        B, H = codes[0].shape[:2]
        rep = H // kv_heads
        codes = (codes[0], np.repeat(codes[1], rep, axis=1), np.repeat(codes[2], rep, axis=1))
        scales = (scales[0], np.repeat(scales[1], rep, axis=1), np.repeat(scales[2], rep, axis=1))
    deq = [_f8.dequantize(c, s, 128) for c, s in zip(codes, scales)]
    B, H, N, d = codes[0].shape
    if rows is None:
        rows = np.arange(B * H * N, dtype=np.int64)
        o_ref, l_ref = _oracle.attention_fwd(*deq, scale, causal)
        o_ref, l_ref = o_ref.reshape(-1, d), l_ref.reshape(-1)
    else:
        o_ref, l_ref = _oracle.attention_fwd_rows(*deq, rows, scale, causal)
    got, got_l = gpu_rows(o, rows), gpu_rows(lse, rows)
    assert np.isfinite(got).all() and np.isfinite(got_l).all()
    bound = fp8_rounding_bound(deq[0], deq[1], _f8.e4m3_decode(codes[2]), scales[2], rows, scale, causal)
    err = np.abs(got - o_ref)
    worst = np.unravel_index(np.argmax(err - 1.02 * bound - 2.0 ** -8 * np.abs(o_ref)), err.shape)
    assert (err <= 1.02 * bound + 2.0 ** -8 * np.abs(o_ref) + 1e-6).all(), \
        (int(rows[worst[0]]), int(worst[1]), float(err[worst]), float(bound[worst]), float(o_ref[worst]))
    assert max_abs(got_l, l_ref) <= 2e-3
    return got, o_ref
