"""ctypes binding over libfa_mi355.so: same names as the C ABI, argument marshalling only.

Every step of the attention path runs in the library's HIP kernels; PyTorch is used here
for device memory and streams.  There is no fallback: if the library has not been built
(`python -m paper_2407_08608_amd.build`), importing a symbol raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfa_mi355.so")

FA_OK = 0
FA_F32, FA_BF16, FA_F16, FA_FP8_E4M3 = 0, 1, 2, 3
_DTYPE_CODE = {torch.float32: FA_F32, torch.bfloat16: FA_BF16, torch.float16: FA_F16}

EXPORTS = ("fa_fwd", "fa_fwd_fp8", "fa_fp8_quant_hadamard", "fa_bwd_workspace_bytes", "fa_bwd",
           "fa_fwd_schedule", "fa_fwd_gqa", "fa_fwd_fp8_gqa", "fa_bwd_gqa", "fa_bwd_noalloc", "fa_fwd_kernel_name",
           "fa_probe_mfma_flops", "fa_probe_mfma", "fa_status_string")

_lib = None


class FaError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: fa_status {status} ({status_string(status)})")


def lib():
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2407_08608_amd.build`; "
                               "there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, fp, ci, cf = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.fa_fwd.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_fwd.restype = ci
        L.fa_fwd_fp8.argtypes = [vp, vp, vp, fp, fp, fp, vp, fp, ci, ci, ci, ci, ci, cf, ci, vp]
        L.fa_fwd_fp8.restype = ci
        L.fa_fp8_quant_hadamard.argtypes = [vp, ci, vp, fp, ci, ci, ci, ci, ci, vp, ci, vp]
        L.fa_fp8_quant_hadamard.restype = ci
        L.fa_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        L.fa_bwd_workspace_bytes.restype = ctypes.c_size_t
        L.fa_bwd.argtypes = [vp] * 10 + [ctypes.c_size_t, ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_bwd.restype = ci
        L.fa_fwd_schedule.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, cf, ci, ci, ci, vp]
        L.fa_fwd_schedule.restype = ci
        L.fa_fwd_gqa.argtypes = [vp, vp, vp, vp, fp, ci, ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_fwd_gqa.restype = ci
        L.fa_fwd_fp8_gqa.argtypes = [vp, vp, vp, fp, fp, fp, vp, fp, ci, ci, ci, ci, ci, ci, cf, ci, vp]
        L.fa_fwd_fp8_gqa.restype = ci
        L.fa_bwd_gqa.argtypes = [vp] * 10 + [ctypes.c_size_t, ci, ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_bwd_gqa.restype = ci
        L.fa_bwd_noalloc.argtypes = [vp] * 9 + [ci, ci, ci, ci, cf, ci, ci, vp]
        L.fa_bwd_noalloc.restype = ci
        L.fa_fwd_kernel_name.argtypes = [ci, ci, ci, ci]
        L.fa_fwd_kernel_name.restype = ctypes.c_char_p
        L.fa_probe_mfma_flops.argtypes = [ci, ci]
        L.fa_probe_mfma_flops.restype = ctypes.c_double
        L.fa_probe_mfma.argtypes = [vp, ctypes.c_size_t, fp, ci, ci, vp]
        L.fa_probe_mfma.restype = ci
        L.fa_status_string.argtypes = [ci]
        L.fa_status_string.restype = ctypes.c_char_p
        _lib = L
    return _lib


def status_string(status):
    return lib().fa_status_string(int(status)).decode()


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check_dev(*ts):
    for t in ts:
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError("tensors must be contiguous device tensors")


def fa_fwd(q, k, v, scale, causal, o=None, lse=None, dtype=None):
    """O, L = attention forward.  q, k, v: [B,H,N,d] device tensors of one dtype
    (float32 / bfloat16 / float16, or uint8 e4m3 codes with dtype=FA_FP8_E4M3)."""
    _check_dev(q, k, v, o, lse)
    B, H, N, d = q.shape
    code = dtype if dtype is not None else _DTYPE_CODE[q.dtype]
    if o is None:
        o = torch.empty((B, H, N, d), device=q.device, dtype=torch.bfloat16 if code == FA_FP8_E4M3 else q.dtype)
    if lse is None:
        lse = torch.empty((B, H, N), device=q.device, dtype=torch.float32)
    st = lib().fa_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d,
                      float(scale), int(bool(causal)), code, _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fwd")
    return o, lse


def fa_fp8_quant_hadamard(x, signs=None, block_rows=128, per_tensor=False, x8=None, scales=None):
    """codes (uint8 e4m3) and per-block scales of x [B,H,N,d]; signs: int8 [d] device tensor or None."""
    _check_dev(x, signs, x8, scales)
    B, H, N, d = x.shape
    nb = -(-N // block_rows)
    if x8 is None:
        x8 = torch.empty((B, H, N, d), device=x.device, dtype=torch.uint8)
    if scales is None:
        scales = torch.empty((B, H, nb), device=x.device, dtype=torch.float32)
    st = lib().fa_fp8_quant_hadamard(x.data_ptr(), _DTYPE_CODE[x.dtype], x8.data_ptr(), scales.data_ptr(), B, H, N, d,
                                     int(block_rows), None if signs is None else signs.data_ptr(),
                                     int(bool(per_tensor)), _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fp8_quant_hadamard")
    return x8, scales


def fa_fwd_fp8(q8, k8, v8, q_scale, k_scale, v_scale, scale, causal, block_rows=128, o=None, lse=None):
    """O (bf16), L from e4m3 codes with per-block scales."""
    _check_dev(q8, k8, v8, q_scale, k_scale, v_scale, o, lse)
    B, H, N, d = q8.shape
    if o is None:
        o = torch.empty((B, H, N, d), device=q8.device, dtype=torch.bfloat16)
    if lse is None:
        lse = torch.empty((B, H, N), device=q8.device, dtype=torch.float32)
    st = lib().fa_fwd_fp8(q8.data_ptr(), k8.data_ptr(), v8.data_ptr(), q_scale.data_ptr(), k_scale.data_ptr(),
                          v_scale.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d, int(block_rows),
                          float(scale), int(bool(causal)), _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fwd_fp8")
    return o, lse


def fa_bwd_workspace_bytes(B, H, N, d, dtype=FA_BF16):
    return int(lib().fa_bwd_workspace_bytes(B, H, N, d, dtype))


def fa_bwd(q, k, v, o, lse, dout, scale, causal, dq=None, dk=None, dv=None, workspace=None):
    """dQ, dK, dV from the forward's inputs, O, L and dO."""
    _check_dev(q, k, v, o, lse, dout, dq, dk, dv, workspace)
    B, H, N, d = q.shape
    code = _DTYPE_CODE[q.dtype]
    need = fa_bwd_workspace_bytes(B, H, N, d, code)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), device=q.device, dtype=torch.uint8)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    st = lib().fa_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), dout.data_ptr(),
                      dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(), workspace.numel(),
                      B, H, N, d, float(scale), int(bool(causal)), code, _stream())
    if st != FA_OK:
        raise FaError(st, "fa_bwd")
    return dq, dk, dv


FA_BWD_NOALLOC_MAX_ROWS = 1048576


def fa_bwd_noalloc(q, k, v, o, lse, dout, scale, causal, dq, dk, dv):
    """fa_bwd on the library's fixed scratch: the caller passes every tensor, outputs included, and the
    call allocates nothing (neither here nor in the library)."""
    _check_dev(q, k, v, o, lse, dout, dq, dk, dv)
    B, H, N, d = q.shape
    st = lib().fa_bwd_noalloc(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), dout.data_ptr(),
                              dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), B, H, N, d, float(scale),
                              int(bool(causal)), _DTYPE_CODE[q.dtype], _stream())
    if st != FA_OK:
        raise FaError(st, "fa_bwd_noalloc")
    return dq, dk, dv


FA_SCHED_AUTO, FA_SCHED_LOCKSTEP_4W, FA_SCHED_LOCKSTEP_8W, FA_SCHED_PINGPONG = 0, 1, 2, 3


def fa_fwd_schedule(q, k, v, scale, causal, schedule, o=None, lse=None):
    """fa_fwd with the kernel schedule forced (ablation)."""
    _check_dev(q, k, v, o, lse)
    B, H, N, d = q.shape
    o = torch.empty_like(q) if o is None else o
    if lse is None:
        lse = torch.empty((B, H, N), device=q.device, dtype=torch.float32)
    st = lib().fa_fwd_schedule(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, N, d,
                               float(scale), int(bool(causal)), _DTYPE_CODE[q.dtype], int(schedule), _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fwd_schedule")
    return o, lse


def fa_fwd_gqa(q, k, v, scale, causal, o=None, lse=None, dtype=None):
    """Grouped-query forward: q [B,H,N,d]; k, v [B,H_kv,N,d] with H_kv dividing H."""
    _check_dev(q, k, v, o, lse)
    B, H, N, d = q.shape
    H_kv = k.shape[1]
    code = dtype if dtype is not None else _DTYPE_CODE[q.dtype]
    if o is None:
        o = torch.empty((B, H, N, d), device=q.device, dtype=torch.bfloat16 if code == FA_FP8_E4M3 else q.dtype)
    if lse is None:
        lse = torch.empty((B, H, N), device=q.device, dtype=torch.float32)
    st = lib().fa_fwd_gqa(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, H_kv, N, d,
                          float(scale), int(bool(causal)), code, _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fwd_gqa")
    return o, lse


def fa_fwd_fp8_gqa(q8, k8, v8, q_scale, k_scale, v_scale, scale, causal, block_rows=128, o=None, lse=None):
    """Grouped-query FP8 forward: q8 [B,H,N,d]; k8, v8 [B,H_kv,N,d] and their scales [B,H_kv,blocks]."""
    _check_dev(q8, k8, v8, q_scale, k_scale, v_scale, o, lse)
    B, H, N, d = q8.shape
    H_kv = k8.shape[1]
    if o is None:
        o = torch.empty((B, H, N, d), device=q8.device, dtype=torch.bfloat16)
    if lse is None:
        lse = torch.empty((B, H, N), device=q8.device, dtype=torch.float32)
    st = lib().fa_fwd_fp8_gqa(q8.data_ptr(), k8.data_ptr(), v8.data_ptr(), q_scale.data_ptr(), k_scale.data_ptr(),
                              v_scale.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H, H_kv, N, d, int(block_rows),
                              float(scale), int(bool(causal)), _stream())
    if st != FA_OK:
        raise FaError(st, "fa_fwd_fp8_gqa")
    return o, lse


def fa_bwd_gqa(q, k, v, o, lse, dout, scale, causal, dq=None, dk=None, dv=None, workspace=None):
    """Grouped-query backward: dQ [B,H,N,d]; dK, dV [B,H_kv,N,d] (summed over each group's query heads)."""
    _check_dev(q, k, v, o, lse, dout, dq, dk, dv, workspace)
    B, H, N, d = q.shape
    H_kv = k.shape[1]
    code = _DTYPE_CODE[q.dtype]
    need = fa_bwd_workspace_bytes(B, H, N, d, code)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), device=q.device, dtype=torch.uint8)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(v) if dv is None else dv
    st = lib().fa_bwd_gqa(q.data_ptr(), k.data_ptr(), v.data_ptr(), o.data_ptr(), lse.data_ptr(), dout.data_ptr(),
                          dq.data_ptr(), dk.data_ptr(), dv.data_ptr(), workspace.data_ptr(), workspace.numel(),
                          B, H, H_kv, N, d, float(scale), int(bool(causal)), code, _stream())
    if st != FA_OK:
        raise FaError(st, "fa_bwd_gqa")
    return dq, dk, dv


def fa_probe_mfma_flops(dtype, iters):
    return float(lib().fa_probe_mfma_flops(int(dtype), int(iters)))


def fa_probe_mfma(operands, dtype, iters, sink=None):
    """One launch of the MFMA-only rate probe on the raw operand bits in `operands` (uint8)."""
    _check_dev(operands, sink)
    if sink is None:
        sink = torch.empty((512,), device=operands.device, dtype=torch.float32)
    st = lib().fa_probe_mfma(operands.data_ptr(), operands.numel() * operands.element_size(), sink.data_ptr(),
                             int(dtype), int(iters), _stream())
    if st != FA_OK:
        raise FaError(st, "fa_probe_mfma")
    return sink


def fa_fwd_kernel_name(dtype, N, d, causal):
    """Profiler name of the kernel that serves this forward request (None if unsupported)."""
    name = lib().fa_fwd_kernel_name(int(dtype), int(N), int(d), int(bool(causal)))
    return None if name is None else name.decode()
