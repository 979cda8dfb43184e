// C ABI of libfa_mi355.so: argument validation and dispatch.  See include/fa_mi355.h for the
// contract of every entry point.
#include <math.h>
#include <stdint.h>

#include <atomic>

#include "fa_launch.h"

// Scratch of fa_bwd_noalloc: the backward's D = rowsum(dO o O) vector.  A file-scope device array, so
// every GPU the library runs on holds its own copy from the moment the code object is loaded until the
// process ends, and no call ever allocates.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels and launches take the per-device address kept in g_scratch_ptr.
static __device__ __align__(256) unsigned char fa_noalloc_scratch[FA_BWD_NOALLOC_MAX_ROWS * sizeof(float)];

namespace {

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Address of the scratch array on the current device (resolved once per device), or nullptr.
void* noalloc_scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(fa_noalloc_scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool head_dim_ok(int d) { return d == 64 || d == 128 || d == 256; }

// A sticky error left on this thread by earlier, unrelated HIP work would otherwise be reported by the
// first hipGetLastError() after our own launch and be mistaken for ours.
void forget_stale_hip_error() { (void)hipGetLastError(); }

int check_common(int B, int H, int N, int d, float scale, int causal) {
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0) return FA_ERR_SHAPE;
    if (!(scale > 0.f) || !isfinite(scale)) return FA_ERR_SHAPE;
    if (causal != 0 && causal != 1) return FA_ERR_SHAPE;
    if ((long)B * H * N > 0x7fffffffL) return FA_ERR_SHAPE;
    if (!head_dim_ok(d)) return FA_ERR_UNSUPPORTED;
    // one head of a tensor is addressed through a 32-bit buffer offset (4 bytes per element at most,
    // and the staging loads run a few blocks past the end)
    if ((long)N * d * 4 > 0x7ff00000L) return FA_ERR_UNSUPPORTED;
    return FA_OK;
}

}  // namespace

extern "C" {

const char* fa_status_string(int status) {
    switch (status) {
        case FA_OK: return "ok";
        case FA_ERR_NULL: return "a required pointer is NULL";
        case FA_ERR_SHAPE: return "invalid shape, scale or flag";
        case FA_ERR_DTYPE: return "unknown dtype";
        case FA_ERR_UNSUPPORTED: return "valid request with no kernel in this build";
        case FA_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
        case FA_ERR_WORKSPACE: return "workspace missing or too small";
        case FA_ERR_LAUNCH: return "HIP runtime rejected the launch";
        case FA_ERR_TOO_LARGE: return "problem exceeds the fixed scratch of an entry point that cannot allocate";
        default: return "unknown status";
    }
}

static int fwd_any(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N,
                   int d, float scale, int causal, int dtype, int schedule, void* stream) {
    if (!q || !k || !v || !o || !lse) return FA_ERR_NULL;
    if (dtype < FA_F32 || dtype > FA_FP8_E4M3) return FA_ERR_DTYPE;
    int st = check_common(B, H, N, d, scale, causal);
    if (st != FA_OK) return st;
    if (H_kv <= 0 || H % H_kv != 0) return FA_ERR_SHAPE;
    if (schedule < FA_SCHED_AUTO || schedule > FA_SCHED_PINGPONG) return FA_ERR_SHAPE;
    if (schedule != FA_SCHED_AUTO && dtype != FA_BF16 && dtype != FA_F16) return FA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse)) return FA_ERR_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    forget_stale_hip_error();
    switch (dtype) {
        case FA_F32: return fa::launch_fwd_f32(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, s);
        case FA_BF16: return fa::launch_fwd_bf16(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, schedule, s);
        case FA_F16: return fa::launch_fwd_f16(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, schedule, s);
        default:
            return fa::launch_fwd_fp8(q, k, v, nullptr, nullptr, nullptr, o, lse, B, H, H_kv, N, d, scale, causal, s);
    }
}

static int fwd_fp8_any(const void* q8, const void* k8, const void* v8, const float* q_scale, const float* k_scale,
                       const float* v_scale, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                       int block_rows, float scale, int causal, void* stream) {
    if (!q8 || !k8 || !v8 || !q_scale || !k_scale || !v_scale || !o || !lse) return FA_ERR_NULL;
    int st = check_common(B, H, N, d, scale, causal);
    if (st != FA_OK) return st;
    if (block_rows <= 0 || H_kv <= 0 || H % H_kv != 0) return FA_ERR_SHAPE;
    if (block_rows != 128) return FA_ERR_UNSUPPORTED;
    if (!aligned16(q8) || !aligned16(k8) || !aligned16(v8) || !aligned16(o) || !aligned16(lse)) return FA_ERR_ALIGN;
    forget_stale_hip_error();
    return fa::launch_fwd_fp8(q8, k8, v8, q_scale, k_scale, v_scale, o, lse, B, H, H_kv, N, d, scale, causal,
                              static_cast<hipStream_t>(stream));
}

int fa_fwd(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d, float scale,
           int causal, int dtype, void* stream) {
    return fwd_any(q, k, v, o, lse, B, H, H, N, d, scale, causal, dtype, FA_SCHED_AUTO, stream);
}

int fa_fwd_schedule(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int N, int d,
                    float scale, int causal, int dtype, int schedule, void* stream) {
    return fwd_any(q, k, v, o, lse, B, H, H, N, d, scale, causal, dtype, schedule, stream);
}

const char* fa_fwd_kernel_name(int dtype, int N, int d, int causal) {
    if (N <= 0 || (causal != 0 && causal != 1)) return nullptr;
    switch (dtype) {
        case FA_F32: return d == 64 ? (causal ? "fa_fwd_f32_kernel<64, 32, true>" : "fa_fwd_f32_kernel<64, 32, false>") : nullptr;
        case FA_BF16: return fa::fwd_16bit_kernel_name(false, N, d, causal);
        case FA_F16: return fa::fwd_16bit_kernel_name(true, N, d, causal);
        case FA_FP8_E4M3: return fa::fwd_fp8_kernel_name(N, d, causal);
        default: return nullptr;
    }
}

int fa_fwd_gqa(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
               float scale, int causal, int dtype, void* stream) {
    return fwd_any(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, dtype, FA_SCHED_AUTO, stream);
}

int fa_fwd_fp8(const void* q8, const void* k8, const void* v8, const float* q_scale, const float* k_scale,
               const float* v_scale, void* o, float* lse, int B, int H, int N, int d, int block_rows, float scale,
               int causal, void* stream) {
    return fwd_fp8_any(q8, k8, v8, q_scale, k_scale, v_scale, o, lse, B, H, H, N, d, block_rows, scale, causal, stream);
}

int fa_fwd_fp8_gqa(const void* q8, const void* k8, const void* v8, const float* q_scale, const float* k_scale,
                   const float* v_scale, void* o, float* lse, int B, int H, int H_kv, int N, int d, int block_rows,
                   float scale, int causal, void* stream) {
    return fwd_fp8_any(q8, k8, v8, q_scale, k_scale, v_scale, o, lse, B, H, H_kv, N, d, block_rows, scale, causal,
                       stream);
}

int fa_fp8_quant_hadamard(const void* x, int in_dtype, void* x8, float* scales, int B, int H, int N, int d,
                          int block_rows, const signed char* signs, int per_tensor, void* stream) {
    if (!x || !x8 || !scales) return FA_ERR_NULL;
    if (in_dtype < FA_F32 || in_dtype > FA_FP8_E4M3) return FA_ERR_DTYPE;
    if (in_dtype == FA_FP8_E4M3) return FA_ERR_UNSUPPORTED;
    if (B <= 0 || H <= 0 || N <= 0 || d <= 0 || block_rows <= 0) return FA_ERR_SHAPE;
    if (per_tensor != 0 && per_tensor != 1) return FA_ERR_SHAPE;
    if ((long)B * H * N > 0x7fffffffL) return FA_ERR_SHAPE;
    if (!head_dim_ok(d) || block_rows != 128) return FA_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(x8)) return FA_ERR_ALIGN;
    forget_stale_hip_error();
    return fa::launch_quant_hadamard(x, in_dtype, x8, scales, B, H, N, d, signs, per_tensor,
                                     static_cast<hipStream_t>(stream));
}

size_t fa_bwd_workspace_bytes(int B, int H, int N, int d, int dtype) {
    if (B <= 0 || H <= 0 || N <= 0 || !head_dim_ok(d)) return 0;
    if (dtype != FA_BF16 && dtype != FA_F16) return 0;
    return fa::bwd_workspace_bytes(B, H, N, d);
}

// Everything about a backward request except its workspace.
static int check_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
                     void* dq, void* dk, void* dv, int B, int H, int H_kv, int N, int d, float scale, int causal,
                     int dtype) {
    if (!q || !k || !v || !o || !lse || !dout || !dq || !dk || !dv) return FA_ERR_NULL;
    if (dtype < FA_F32 || dtype > FA_FP8_E4M3) return FA_ERR_DTYPE;
    int st = check_common(B, H, N, d, scale, causal);
    if (st != FA_OK) return st;
    if (H_kv <= 0 || H % H_kv != 0) return FA_ERR_SHAPE;
    if (dtype != FA_BF16 && dtype != FA_F16) return FA_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(lse) || !aligned16(dout) ||
        !aligned16(dq) || !aligned16(dk) || !aligned16(dv))
        return FA_ERR_ALIGN;
    return FA_OK;
}

static int bwd_any(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
                   void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, int B, int H, int H_kv, int N,
                   int d, float scale, int causal, int dtype, void* stream) {
    int st = check_bwd(q, k, v, o, lse, dout, dq, dk, dv, B, H, H_kv, N, d, scale, causal, dtype);
    if (st != FA_OK) return st;
    if (!workspace || workspace_bytes < fa::bwd_workspace_bytes(B, H, N, d)) return FA_ERR_WORKSPACE;
    if (!aligned16(workspace)) return FA_ERR_ALIGN;
    forget_stale_hip_error();
    return fa::launch_bwd(q, k, v, o, lse, dout, dq, dk, dv, workspace, B, H, H_kv, N, d, scale, causal, dtype,
                          static_cast<hipStream_t>(stream));
}

int fa_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout, void* dq,
           void* dk, void* dv, void* workspace, size_t workspace_bytes, int B, int H, int N, int d, float scale,
           int causal, int dtype, void* stream) {
    return bwd_any(q, k, v, o, lse, dout, dq, dk, dv, workspace, workspace_bytes, B, H, H, N, d, scale, causal, dtype,
                   stream);
}

int fa_bwd_gqa(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
               void* dq, void* dk, void* dv, void* workspace, size_t workspace_bytes, int B, int H, int H_kv, int N,
               int d, float scale, int causal, int dtype, void* stream) {
    return bwd_any(q, k, v, o, lse, dout, dq, dk, dv, workspace, workspace_bytes, B, H, H_kv, N, d, scale, causal,
                   dtype, stream);
}

int fa_bwd_noalloc(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
                   void* dq, void* dk, void* dv, int B, int H, int N, int d, float scale, int causal, int dtype,
                   void* stream) {
    int st = check_bwd(q, k, v, o, lse, dout, dq, dk, dv, B, H, H, N, d, scale, causal, dtype);
    if (st != FA_OK) return st;
    if ((long)B * H * N > (long)FA_BWD_NOALLOC_MAX_ROWS) return FA_ERR_TOO_LARGE;
    forget_stale_hip_error();
    void* scratch = noalloc_scratch_on_current_device();
    if (!scratch) return FA_ERR_LAUNCH;
    // D is written in full by the first kernel before the others read it: nothing to clear
    return fa::launch_bwd(q, k, v, o, lse, dout, dq, dk, dv, scratch, B, H, H, N, d, scale, causal, dtype,
                          static_cast<hipStream_t>(stream));
}

double fa_probe_mfma_flops(int dtype, int iters) {
    if ((dtype != FA_BF16 && dtype != FA_FP8_E4M3) || iters <= 0) return 0.0;
    return fa::probe_mfma_flops(iters, dtype == FA_FP8_E4M3);
}

int fa_probe_mfma(const void* operands, size_t operand_bytes, float* sink, int dtype, int iters, void* stream) {
    if (!operands || !sink) return FA_ERR_NULL;
    if (dtype < FA_F32 || dtype > FA_FP8_E4M3) return FA_ERR_DTYPE;
    if (dtype != FA_BF16 && dtype != FA_FP8_E4M3) return FA_ERR_UNSUPPORTED;
    if (operand_bytes < 16 || operand_bytes % 16 != 0 || operand_bytes > (size_t)1 << 30 || iters <= 0 || iters > 1000000)
        return FA_ERR_SHAPE;
    if (!aligned16(operands) || !aligned16(sink)) return FA_ERR_ALIGN;
    forget_stale_hip_error();
    return fa::launch_probe_mfma(operands, operand_bytes, sink, iters, dtype == FA_FP8_E4M3,
                                 static_cast<hipStream_t>(stream));
}

}  // extern "C"
