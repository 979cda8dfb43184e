/*
 * fa_mi355 -- exact fused scaled-dot-product attention for AMD MI355X (gfx950).
 *
 * C ABI of libfa_mi355.so.  The operation is the one stated in section 2.1 of the
 * FlashAttention-3 paper (arXiv 2407.08608):
 *
 *     S = scale * Q K^T,   P = softmax_rows(S [causal: keys j > i masked]),   O = P V,
 *
 * computed per (batch, head) without ever materialising S or P (Algorithm 1: tiled
 * Q K^T, online softmax with running row maximum / row sum, P V accumulated on chip),
 * and the row-wise logsumexp  L_i = m_i + log(l_i)  written out for the backward pass.
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers owned by the caller.  The library reads
 *     inputs, writes outputs, and keeps no reference after the call returns.
 *   - Tensors are contiguous [B, H, N, d] with d fastest (paper section 3.3: inputs are
 *     contiguous in the head dimension); lse / D-like vectors are fp32 [B, H, N].
 *     Every tensor pointer must be 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *     asynchronous with respect to the host: they enqueue kernels and return.  They
 *     never synchronise, allocate or free device memory, throw, or abort.
 *   - The return value is an fa_status.  Every argument and size check precedes the first
 *     launch: on any status other than FA_OK and FA_ERR_LAUNCH nothing has been enqueued.
 *     FA_ERR_LAUNCH means the HIP runtime refused a launch; calls made of several kernels
 *     (fa_bwd*: three, fa_fp8_quant_hadamard with per_tensor = 1: four) stop at the refused
 *     one, and the outputs are then undefined.  fa_status_string() names a status.
 *   - Supported head dimensions: d in {64, 128, 256}.  N >= 1 (any N; rows past N are
 *     never read or written).  B, H >= 1.  scale finite and > 0.  causal in {0, 1};
 *     causal means key j is visible to query i iff j <= i (N_q == N_k).
 *   - Size limits: B*H*N < 2^31 rows (else FA_ERR_SHAPE) and, because one head is
 *     addressed through 32-bit byte offsets, 4*N*d <= 0x7ff00000 (else
 *     FA_ERR_UNSUPPORTED): N <= 4 192 256 at d = 128, twice that at d = 64, half at 256.
 *   - Thread-safe: no mutable global state.
 */
#ifndef FA_MI355_H
#define FA_MI355_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FA_OK = 0,
    FA_ERR_NULL = 1,        /* a required pointer is NULL */
    FA_ERR_SHAPE = 2,       /* B, H, N or block_rows not positive, scale not finite/positive, causal not 0/1 */
    FA_ERR_DTYPE = 3,       /* dtype is not a member of fa_dtype */
    FA_ERR_UNSUPPORTED = 4, /* a valid request this build has no kernel for (e.g. head dim 96) */
    FA_ERR_ALIGN = 5,       /* a tensor pointer is not 16-byte aligned */
    FA_ERR_WORKSPACE = 6,   /* workspace NULL or smaller than fa_bwd_workspace_bytes() */
    FA_ERR_LAUNCH = 7,      /* the HIP runtime rejected a launch */
    FA_ERR_TOO_LARGE = 8    /* fa_bwd_noalloc: B*H*N exceeds FA_BWD_NOALLOC_MAX_ROWS */
} fa_status;

typedef enum {
    FA_F32 = 0,     /* fp32 in / fp32 out, fp32 arithmetic (d = 64 only) */
    FA_BF16 = 1,    /* bf16 in / bf16 out, fp32 accumulate */
    FA_F16 = 2,     /* fp16 in / fp16 out, fp32 accumulate */
    FA_FP8_E4M3 = 3 /* OCP e4m3 ("fn") codes in, bf16 out, fp32 accumulate */
} fa_dtype;

/*
 * Forward pass (section 2.1; Algorithms 1 and 2).
 *   q, k, v : [B,H,N,d] of `dtype`            (device, read)
 *   o       : [B,H,N,d] of `dtype` (bf16 when dtype == FA_FP8_E4M3)   (device, written)
 *   lse     : fp32 [B,H,N], natural log of sum_j exp(scale * q_i . k_j) over visible j
 *             (device, written)
 * With dtype == FA_FP8_E4M3 the codes are taken at unit scale (the block-scaled path is
 * fa_fwd_fp8).  FA_F32 supports d = 64 only.
 */
int fa_fwd(const void* q, const void* k, const void* v, void* o, float* lse,
           int B, int H, int N, int d, float scale, int causal, int dtype, void* stream);

/*
 * FP8 forward with per-block scales (section 3.3, "block quantization": one scalar per
 * block of rows of Q, K and V; each block of S is rescaled by the product of its Q-block
 * and K-block scales at no extra cost).
 *   q8, k8, v8 : e4m3 codes [B,H,N,d]                         (device, read)
 *   q_scale, k_scale, v_scale : fp32 [B,H,ceil(N/block_rows)]; the real tensor is
 *             code * scale of its block                        (device, read).  Every scale must
 *             be finite and > 0 (an all-zero block carries scale 1, as fa_fp8_quant_hadamard
 *             writes it): log2(v_scale) and 1 / v_scale enter the row maximum and the row sum,
 *             so a zero, negative or non-finite scale gives NaN rows.  Not checked (the values
 *             live on the device).
 *   o   : bf16 [B,H,N,d]; lse : fp32 [B,H,N]                   (device, written)
 *   block_rows : rows per quantisation block; must be 128.
 * Q and K are expected to have been multiplied by the same orthogonal matrix
 * ("incoherent processing"); the kernel neither knows nor cares, since (QM)(KM)^T = QK^T.
 */
int fa_fwd_fp8(const void* q8, const void* k8, const void* v8,
               const float* q_scale, const float* k_scale, const float* v_scale,
               void* o, float* lse, int B, int H, int N, int d, int block_rows,
               float scale, int causal, void* stream);

/*
 * Quantisation pre-pass (section 3.3: block quantization + incoherent processing).
 * Row-wise  y = (x * signs) H_d / sqrt(d)  with H_d the Sylvester Hadamard matrix
 * (skipped when signs == NULL), then per block of `block_rows` rows of one head:
 *     scale = amax|y| / 448  (1 if the block is all zero),
 *     code  = round-to-nearest-even e4m3 of clamp(y * (448 / amax), +-448).
 *   x       : [B,H,N,d] of in_dtype (FA_F32, FA_BF16 or FA_F16)   (device, read)
 *   x8      : e4m3 codes [B,H,N,d]                                (device, written)
 *   scales  : fp32 [B,H,ceil(N/block_rows)]                        (device, written)
 *   signs   : int8 [d] of +1 / -1, or NULL for no transform        (device, read)
 *   per_tensor : 0 = per-block scales; 1 = one scale from the amax of the whole
 *             transformed tensor, replicated into every slot of `scales` (the per-tensor
 *             baseline of section 4.3).  In this mode `scales` is also used as scratch
 *             during the call.
 *   block_rows must be 128.
 */
int fa_fp8_quant_hadamard(const void* x, int in_dtype, void* x8, float* scales,
                          int B, int H, int N, int d, int block_rows,
                          const signed char* signs, int per_tensor, void* stream);

/*
 * Backward pass (section 2.1 chain rule; recomputation of P from L as in Algorithm 3):
 *     D = rowsum(dO o O);  P = exp(S - L);  dV = P^T dO;  dP = dO V^T;
 *     dS = P o (dP - D);   dQ = scale * dS K;   dK = scale * dS^T Q.
 *   q, k, v, o, dout : [B,H,N,d] of `dtype`; lse : fp32 [B,H,N] from fa_fwd   (device, read)
 *   dq, dk, dv       : [B,H,N,d] of `dtype`                                   (device, written)
 *   workspace        : device scratch of at least fa_bwd_workspace_bytes(...) bytes (it holds D),
 *                      16-byte aligned, owned by the caller, contents undefined on return.
 * dtype FA_BF16 or FA_F16 (others: FA_ERR_UNSUPPORTED; fa_bwd_workspace_bytes then returns 0);
 * d = 64, 128 or 256.  Nothing is accumulated
 * with atomics: results are bit-for-bit repeatable.
 */
size_t fa_bwd_workspace_bytes(int B, int H, int N, int d, int dtype);

int fa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse,
           const void* dout, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
           int B, int H, int N, int d, float scale, int causal, int dtype, void* stream);

/*
 * fa_bwd for callers that cannot allocate or hand over device scratch: code running under HIP
 * graph capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same
 * operation, arguments, kernels and results (bit for bit) as fa_bwd, but the D vector lives in a
 * fixed device array inside the library instead of a caller workspace; the call allocates and frees
 * nothing.
 *   - Limit: B*H*N <= FA_BWD_NOALLOC_MAX_ROWS (4 MiB of scratch per GPU, held by every GPU the
 *     library is used on until the process ends); larger requests return FA_ERR_TOO_LARGE and
 *     launch nothing.
 *   - The array is per GPU and shared by every call on that GPU: two calls that may run
 *     concurrently on one GPU (different streams, different host threads) race on it and must be
 *     serialised by the caller; calls on one stream are ordered and safe.  Nothing in it needs
 *     clearing between calls (the first kernel of a call overwrites what the others read).
 *   - The array's device address is looked up once per GPU on the first call made with that GPU
 *     current; if that lookup fails the call returns FA_ERR_LAUNCH.
 */
#define FA_BWD_NOALLOC_MAX_ROWS 1048576

int fa_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const float* lse,
                   const void* dout, void* dq, void* dk, void* dv,
                   int B, int H, int N, int d, float scale, int causal, int dtype, void* stream);

/*
 * Forward pass with the kernel schedule forced, for the scheduling ablation (section 4.2,
 * "2-stage pipelining experiments", re-done with this chip's mechanisms).  Same contract as
 * fa_fwd; FA_SCHED_AUTO is fa_fwd itself.  The other values need dtype FA_BF16 or FA_F16 and
 * d = 128 (else FA_ERR_UNSUPPORTED); an unknown value is FA_ERR_SHAPE.
 */
typedef enum {
    FA_SCHED_AUTO = 0,        /* the library's choice by shape */
    FA_SCHED_LOCKSTEP_4W = 1, /* 128-query tile, 4 waves in lock-step, K/V staged through registers;
                                 softmax/GEMM overlap only across two resident workgroups */
    FA_SCHED_LOCKSTEP_8W = 2, /* 256-query tile, 8 waves in lock-step, K/V staged through registers */
    FA_SCHED_PINGPONG = 3     /* 256-query tile, two wave groups alternating GEMMs and softmax,
                                 K/V staged asynchronously into a 4-deep LDS ring */
} fa_schedule;

int fa_fwd_schedule(const void* q, const void* k, const void* v, void* o, float* lse,
                    int B, int H, int N, int d, float scale, int causal, int dtype, int schedule,
                    void* stream);

/*
 * Which kernel serves a forward request: the name a profiler (rocprofv3 --kernel-trace) shows for
 * the kernel that fa_fwd (dtype FA_F32 / FA_BF16 / FA_F16) or fa_fwd_fp8 (dtype FA_FP8_E4M3, the
 * block-scaled instantiation) launches for N keys, head dimension d and this mask.  The choice
 * depends on nothing else.  Host only: launches nothing, touches no device.  Returns a static
 * NUL-terminated string, or NULL for a request those calls would reject.  For measurement code that
 * must attribute launches to kernels without copying the library's thresholds.
 */
const char* fa_fwd_kernel_name(int dtype, int N, int d, int causal);

/*
 * Multi-query / grouped-query attention (section 3.1, "Attention variants": the tensor
 * indexing changes, K and V are not duplicated in HBM).  q, o, dout, dq are [B,H,N,d] and
 * lse is [B,H,N] as above; k, v, dk, dv are [B,H_kv,N,d] (FP8: k_scale, v_scale are
 * [B,H_kv,ceil(N/block_rows)]), with H_kv >= 1 dividing H (else FA_ERR_SHAPE).  Query head h
 * reads key/value head h / (H / H_kv): consecutive query heads form a group.  dk and dv are
 * the sums over the query heads of a group, accumulated on chip in a fixed order (no
 * atomics).  H_kv == H is exactly fa_fwd / fa_fwd_fp8 / fa_bwd.  The workspace size is
 * fa_bwd_workspace_bytes(B, H, N, d, dtype), as for fa_bwd.  Everything else (dtypes, head
 * dimensions, alignment, errors) is as documented for the entry point of the same name
 * without the suffix.
 */
int fa_fwd_gqa(const void* q, const void* k, const void* v, void* o, float* lse,
               int B, int H, int H_kv, int N, int d, float scale, int causal, int dtype, void* stream);

int fa_fwd_fp8_gqa(const void* q8, const void* k8, const void* v8,
                   const float* q_scale, const float* k_scale, const float* v_scale,
                   void* o, float* lse, int B, int H, int H_kv, int N, int d, int block_rows,
                   float scale, int causal, void* stream);

int fa_bwd_gqa(const void* q, const void* k, const void* v, const void* o, const float* lse,
               const void* dout, void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes,
               int B, int H, int H_kv, int N, int d, float scale, int causal, int dtype, void* stream);

/*
 * Measurement aid, not part of the attention path: the rate of the matrix pipes alone.  The
 * roofline fractions of the kernels above are quoted against the published MFMA peak; this
 * call measures what the chip sustains when every wave issues only independent MFMAs
 * (bf16 32x32x16 for FA_BF16, e4m3 32x32x64 for FA_FP8_E4M3) on operand bits of the caller's
 * choosing, which is the practical ceiling for an MFMA-bound kernel on such data.
 *   operands      : device, read; operand_bytes (a multiple of 16, at most 1 GiB) of raw
 *                   operand bits in `dtype`; each lane loads 128 bytes from it once
 *   sink          : device, at least 512 floats; never written in practice (it keeps the
 *                   arithmetic observable)
 *   iters         : 1 .. 1e6 loop trips of 32 MFMAs per wave
 * One launch of 512 workgroups x 8 waves performs fa_probe_mfma_flops(dtype, iters) FLOPs
 * (0.0 for an unsupported dtype or iters <= 0); the caller times it.
 */
double fa_probe_mfma_flops(int dtype, int iters);

int fa_probe_mfma(const void* operands, size_t operand_bytes, float* sink, int dtype, int iters,
                  void* stream);

/* Static, NUL-terminated description of an fa_status value. */
const char* fa_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* FA_MI355_H */
