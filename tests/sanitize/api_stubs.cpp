// Stand-ins for the kernel launchers, so that the argument-validation layer (csrc/fa_api.hip) can be linked and
// run under host sanitizers without any device code: a request that passes validation ends here.
#include "../../paper_2407_08608_amd/csrc/fa_launch.h"

namespace fa {
int launch_fwd_bf16(const void*, const void*, const void*, void*, float*, int, int, int, int, int, float, int, int,
                    hipStream_t) { return FA_OK; }
int launch_fwd_f16(const void*, const void*, const void*, void*, float*, int, int, int, int, int, float, int, int,
                   hipStream_t) { return FA_OK; }
int launch_fwd_f32(const void*, const void*, const void*, void*, float*, int, int, int, int, int, float, int,
                   hipStream_t) { return FA_OK; }
int launch_fwd_fp8(const void*, const void*, const void*, const float*, const float*, const float*, void*, float*, int,
                   int, int, int, int, float, int, hipStream_t) { return FA_OK; }
const char* fwd_16bit_kernel_name(bool, int, int d, int) { return (d == 64 || d == 128 || d == 256) ? "stub" : nullptr; }
const char* fwd_fp8_kernel_name(int, int, int) { return "stub"; }
int launch_quant_hadamard(const void*, int, void*, float*, int, int, int, int, const signed char*, int, hipStream_t) {
    return FA_OK;
}
size_t bwd_workspace_bytes(int B, int H, int N, int) { return (((size_t)B * H * N * sizeof(float)) + 15) & ~(size_t)15; }
int launch_bwd(const void*, const void*, const void*, const void*, const float*, const void*, void*, void*, void*,
               void*, int, int, int, int, int, float, int, int, hipStream_t) { return FA_OK; }
int launch_probe_mfma(const void*, size_t, float*, int, bool, hipStream_t) { return FA_OK; }
double probe_mfma_flops(int iters, bool) { return (double)iters; }
}  // namespace fa
