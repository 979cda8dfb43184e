"""CPU oracle for the FP8 pre-pass: e4m3 codec, sign-diagonal Hadamard transform,
per-block quantisation (paper section 3.3, "block quantization" and "incoherent
processing").

TEST INFRASTRUCTURE ONLY: nothing on the product path may import this module, and it
shares no code with the HIP library.

Readings of the paper taken here (it gives no formulas for any of them):
  * e4m3 is the OCP "fn" flavour: 1 sign, 4 exponent (bias 7), 3 mantissa bits, no
    infinities, S.1111.111 is NaN, largest finite value 448.
  * M = diag(s) * H_d / sqrt(d), H_d the Sylvester Hadamard matrix in natural order, s a
    vector of +-1 supplied by the caller; a row x maps to (x * s) H_d / sqrt(d).
  * One scale per block of `block_rows` consecutive rows of one head:
    scale = amax / 448 (1 if the block is all zero), code = RNE_e4m3(clamp(y * (448 / amax))).
  * The quantisation decision is taken in fp32 (the precision the kernel computes in):
    the transform runs as log2(d) stages of fp32 add/sub butterflies with strides
    1, 2, 4, ..., d/2, then one fp32 multiply by float32(1/sqrt(d)).
"""
import numpy as np

E4M3_MAX = 448.0


def e4m3_decode_table():
    """All 256 code points as float64 (NaN for 0x7F / 0xFF), from the format definition."""
    out = np.empty(256, dtype=np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = np.nan
        elif e == 0:
            out[code] = sign * (m / 8.0) * 2.0 ** (-6)
        else:
            out[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


_TABLE = e4m3_decode_table()
_POS = _TABLE[:127].copy()  # codes 0..126: the non-negative finite values, increasing


def e4m3_decode(codes):
    return _TABLE[np.asarray(codes, dtype=np.uint8)]


def e4m3_encode(x):
    """Round-to-nearest-even onto the e4m3 grid with saturation to +-448.  x: finite floats."""
    x = np.asarray(x, dtype=np.float64)
    a = np.minimum(np.abs(x), E4M3_MAX)
    # nearest grid point: index of the first grid value >= a, then compare with the one below
    hi = np.searchsorted(_POS, a, side="left")
    hi = np.minimum(hi, 126)
    lo = np.maximum(hi - 1, 0)
    d_hi = _POS[hi] - a
    d_lo = a - _POS[lo]
    pick_lo = (d_lo < d_hi) | ((d_lo == d_hi) & (lo % 2 == 0))
    code = np.where(pick_lo, lo, hi).astype(np.uint8)
    neg = np.signbit(x)
    return np.where(neg, code | 0x80, code).astype(np.uint8)


def hadamard_matrix(d):
    """Sylvester construction H_1 = [1], H_2n = [[H, H], [H, -H]] (natural order), float64."""
    assert d >= 1 and (d & (d - 1)) == 0
    Hm = np.ones((1, 1), dtype=np.float64)
    while Hm.shape[0] < d:
        Hm = np.block([[Hm, Hm], [Hm, -Hm]])
    return Hm


def incoherent_matrix(signs):
    """M = diag(s) H_d / sqrt(d) as a dense float64 matrix (orthogonal)."""
    s = np.asarray(signs, dtype=np.float64)
    d = s.shape[0]
    return (s[:, None] * hadamard_matrix(d)) / np.sqrt(d)


def fwht_f32(x):
    """Unnormalised Sylvester transform along the last axis in fp32, strides 1, 2, ..., d/2."""
    y = np.array(x, dtype=np.float32, copy=True)
    d = y.shape[-1]
    assert (d & (d - 1)) == 0
    h = 1
    while h < d:
        y = y.reshape(y.shape[:-1] + (d // (2 * h), 2, h))
        a = y[..., 0, :]
        b = y[..., 1, :]
        y = np.stack([a + b, a - b], axis=-2).astype(np.float32)
        y = y.reshape(y.shape[:-3] + (d,))
        h *= 2
    return y


def transform_f32(x, signs):
    """Row-wise x -> (x * s) H_d / sqrt(d) in fp32 (signs None: identity)."""
    x = np.asarray(x, dtype=np.float32)
    if signs is None:
        return x
    d = x.shape[-1]
    s = np.asarray(signs, dtype=np.float32)
    y = fwht_f32(x * s)
    return (y * np.float32(1.0 / np.sqrt(float(d)))).astype(np.float32)


def quantize(x, signs, block_rows, per_tensor=False):
    """The pre-pass on a [B, H, N, d] float32 array (values of the stored inputs).

    Returns (codes uint8 [B,H,N,d], scales float32 [B,H,ceil(N/block_rows)]).
    per_tensor: one scale from the amax of the whole tensor, replicated into every slot.
    """
    y = transform_f32(x, signs)
    B, H, N, d = y.shape
    nb = -(-N // block_rows)
    scales = np.ones((B, H, nb), dtype=np.float32)
    codes = np.zeros((B, H, N, d), dtype=np.uint8)
    f448 = np.float32(E4M3_MAX)
    tensor_amax = np.float32(np.max(np.abs(y))) if y.size else np.float32(0)
    for b in range(B):
        for h in range(H):
            for t in range(nb):
                blk = y[b, h, t * block_rows:(t + 1) * block_rows]
                amax = tensor_amax if per_tensor else np.float32(np.max(np.abs(blk)))
                if amax == 0:
                    scales[b, h, t] = np.float32(1.0)
                    inv = np.float32(1.0)
                else:
                    scales[b, h, t] = amax / f448
                    inv = f448 / amax
                z = (blk * inv).astype(np.float32)
                z = np.clip(z, -f448, f448)
                codes[b, h, t * block_rows:(t + 1) * block_rows] = e4m3_encode(z)
    return codes, scales


def dequantize(codes, scales, block_rows):
    """codes * scale of the block, float64 [B,H,N,d]."""
    vals = e4m3_decode(codes)
    N = codes.shape[2]
    s = np.repeat(scales.astype(np.float64), block_rows, axis=2)[:, :, :N]
    return vals * s[..., None]
