// Host-side launch entry points, one per kernel family.  H_kv is the number of key/value heads
// (H for ordinary multi-head attention; a divisor of H for multi-query / grouped-query attention).  Each validates nothing (the C ABI
// layer has done that), enqueues on `stream`, and returns an fa_status.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>

#include "../../include/fa_mi355.h"

namespace fa {

int launch_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                    float scale, int causal, int schedule, hipStream_t stream);
int launch_fwd_f16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                   float scale, int causal, int schedule, hipStream_t stream);
int launch_fwd_f32(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                   float scale, int causal, hipStream_t stream);
int launch_fwd_fp8(const void* q8, const void* k8, const void* v8, const float* q_scale, const float* k_scale,
                   const float* v_scale, void* o, float* lse, int B, int H, int H_kv, int N, int d, float scale, int causal,
                   hipStream_t stream);
const char* fwd_16bit_kernel_name(bool f16, int N, int d, int causal);
const char* fwd_fp8_kernel_name(int N, int d, int causal);
int launch_quant_hadamard(const void* x, int in_dtype, void* x8, float* scales, int B, int H, int N, int d,
                          const signed char* signs, int per_tensor, hipStream_t stream);
size_t bwd_workspace_bytes(int B, int H, int N, int d);
int launch_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
               void* dq, void* dk, void* dv, void* workspace, int B, int H, int H_kv, int N, int d, float scale,
               int causal, int dtype, hipStream_t stream);
int launch_probe_mfma(const void* operands, size_t operand_bytes, float* sink, int iters, bool fp8, hipStream_t stream);
double probe_mfma_flops(int iters, bool fp8);

}  // namespace fa
