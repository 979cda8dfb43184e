"""fp64 CPU oracle for the attention path -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu-baseline leg may import this
package.  It wraps `attention_oracle.c` (plain C, fp64, the definition of section 2.1
of the paper written out row by row) through ctypes and holds the numpy FP8 pre-pass
oracle in `fp8_oracle`.  It shares no code with, and never imports, the HIP library.

Every function here takes and returns numpy float64 arrays laid out [B, H, N, d]
(L, D: [B, H, N]).  Callers upcast the stored bf16/fp16/fp32 bits exactly to float64
first, so input rounding is never charged to the kernel under test.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "attention_oracle.c")
_SO = os.path.join(_HERE, "liboracle_attn.so")
_lib = None


def build(force=True):
    """Compile the C oracle with gcc (OpenMP).  Building the checker is not using it."""
    if not force and os.path.exists(_SO) and os.path.getmtime(_SO) >= os.path.getmtime(_SRC):
        return _SO
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", _SO, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_SO)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        ci, cd, cl = ctypes.c_int, ctypes.c_double, ctypes.c_long
        lib.oracle_num_threads.restype = ci
        lib.oracle_attn_fwd.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, cd, ci]
        lib.oracle_attn_fwd.restype = None
        lib.oracle_attn_fwd_rows.argtypes = [dp, dp, dp, ip, cl, dp, dp, ci, ci, ci, ci, cd, ci]
        lib.oracle_attn_fwd_rows.restype = None
        lib.oracle_attn_bwd.argtypes = [dp] * 10 + [ci, ci, ci, ci, cd, ci]
        lib.oracle_attn_bwd.restype = None
        lib.oracle_attn_bwd_dq_rows.argtypes = [dp, dp, dp, dp, ip, cl, dp, ci, ci, ci, ci, cd, ci]
        lib.oracle_attn_bwd_dq_rows.restype = None
        lib.oracle_attn_bwd_dkdv_keys.argtypes = [dp, dp, dp, dp, ci, ci, dp, dp, ci, ci, cd, ci]
        lib.oracle_attn_bwd_dkdv_keys.restype = None
        lib.oracle_attn_probs.argtypes = [dp, dp, dp, dp, ci, ci, cd, ci]
        lib.oracle_attn_probs.restype = None
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def attention_fwd(q, k, v, alpha, causal):
    """O [B,H,N,d] and L [B,H,N] by the definition (section 2.1; L per Algorithm 1's epilogue)."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, N, d = q.shape
    assert k.shape == q.shape and v.shape == q.shape
    o = np.empty_like(q)
    lse = np.empty((B, H, N), dtype=np.float64)
    _load().oracle_attn_fwd(_p(q), _p(k), _p(v), _p(o), _p(lse), B, H, N, d, float(alpha), int(bool(causal)))
    return o, lse


def attention_fwd_rows(q, k, v, rows, alpha, causal):
    """Same, for the flat row indices `rows` (into B*H*N) only: O_rows [n,d], L_rows [n]."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    B, H, N, d = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < B * H * N))
    o = np.empty((rows.size, d), dtype=np.float64)
    lse = np.empty((rows.size,), dtype=np.float64)
    _load().oracle_attn_fwd_rows(_p(q), _p(k), _p(v), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                 rows.size, _p(o), _p(lse), B, H, N, d, float(alpha), int(bool(causal)))
    return o, lse


def attention_bwd(q, k, v, dout, alpha, causal):
    """Gradients by the chain rule of section 2.1.  Returns dict(o, lse, D, dq, dk, dv)."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    o = np.empty_like(q)
    dq = np.empty_like(q)
    dk = np.empty_like(q)
    dv = np.empty_like(q)
    lse = np.empty((B, H, N), dtype=np.float64)
    D = np.empty((B, H, N), dtype=np.float64)
    _load().oracle_attn_bwd(_p(q), _p(k), _p(v), _p(dout), _p(o), _p(lse), _p(D), _p(dq), _p(dk), _p(dv),
                            B, H, N, d, float(alpha), int(bool(causal)))
    return dict(o=o, lse=lse, D=D, dq=dq, dk=dk, dv=dv)


def attention_bwd_dq_rows(q, k, v, dout, rows, alpha, causal):
    """dQ of the flat query rows `rows` (into B*H*N) only, [n,d]: the row-by-row arithmetic of
    `attention_bwd`, for problems too long to differentiate whole."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.ndim == 1 and (rows.size == 0 or (rows.min() >= 0 and rows.max() < B * H * N))
    dq = np.empty((rows.size, d), dtype=np.float64)
    _load().oracle_attn_bwd_dq_rows(_p(q), _p(k), _p(v), _p(dout), rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)),
                                    rows.size, _p(dq), B, H, N, d, float(alpha), int(bool(causal)))
    return dq


def attention_bwd_dkdv_keys(q, k, v, dout, j0, j1, alpha, causal):
    """dK and dV ([j1-j0, d] each) of the key rows j0..j1-1 of a single head (q, k, v, dout: [N,d]).
    Under the causal mask only the queries from j0 on reach these keys, so the last keys of a long
    sequence cost a few full rows."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    N, d = q.shape
    assert 0 <= j0 <= j1 <= N
    dk = np.empty((j1 - j0, d), dtype=np.float64)
    dv = np.empty((j1 - j0, d), dtype=np.float64)
    _load().oracle_attn_bwd_dkdv_keys(_p(q), _p(k), _p(v), _p(dout), int(j0), int(j1), _p(dk), _p(dv), N, d,
                                      float(alpha), int(bool(causal)))
    return dk, dv


def attention_probs(q, k, v, alpha, causal):
    """P [N,N] of a single head (q, k, v: [N,d])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    N, d = q.shape
    P = np.empty((N, N), dtype=np.float64)
    _load().oracle_attn_probs(_p(q), _p(k), _p(v), _p(P), N, d, float(alpha), int(bool(causal)))
    return P


def _expand_kv_heads(x, H):
    """[B,H_kv,N,d] -> [B,H,N,d]: query head h reads key/value head h // (H / H_kv)."""
    H_kv = x.shape[1]
    assert H % H_kv == 0, "the number of query heads must be a multiple of the key/value heads"
    return np.repeat(x, H // H_kv, axis=1)


def attention_fwd_gqa(q, k, v, alpha, causal):
    """Multi-query / grouped-query attention (section 3.1, "Attention variants"): q is [B,H,N,d],
    k and v are [B,H_kv,N,d] with H_kv dividing H; consecutive groups of H/H_kv query heads share
    one key/value head.  By definition this is ordinary attention on K and V repeated per group."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    H = q.shape[1]
    return attention_fwd(q, _expand_kv_heads(k, H), _expand_kv_heads(v, H), alpha, causal)


def attention_bwd_gqa(q, k, v, dout, alpha, causal):
    """Gradients of the grouped-query forward: the repeat of K and V fans each key/value head out to
    H/H_kv query heads, so its gradient is the sum of the per-query-head gradients of that group."""
    q, k, v, dout = _f64(q), _f64(k), _f64(v), _f64(dout)
    B, H, N, d = q.shape
    H_kv = k.shape[1]
    r = attention_bwd(q, _expand_kv_heads(k, H), _expand_kv_heads(v, H), dout, alpha, causal)
    r["dk"] = r["dk"].reshape(B, H_kv, H // H_kv, N, d).sum(axis=2)
    r["dv"] = r["dv"].reshape(B, H_kv, H // H_kv, N, d).sum(axis=2)
    return r
