// Measurement aid: the rate of the matrix pipes alone, on operand bits the caller supplies.
//
// Every wave of a full-chip launch (two workgroups of eight waves per compute unit) loads its
// MFMA operands once and then issues nothing but independent MFMAs.  The attention kernels'
// roofline fractions are quoted against the published peak; this probe shows what part of that
// peak the chip delivers for a given operand bit pattern (the clock drops with the switching
// activity of the operands), which is the ceiling any MFMA-bound kernel here works under.
#include "fa_device.h"
#include "fa_launch.h"

namespace fa {

constexpr int kProbeWgs = 512;
constexpr int kProbeThreads = 512;
constexpr int kProbeUnroll = 32;

template <bool FP8>
__global__ void __launch_bounds__(kProbeThreads, 2)
fa_probe_mfma_kernel(const i32x4* __restrict__ operands, int n_vec, float* __restrict__ sink, int iters) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    i32x4 w[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) w[i] = operands[(threadIdx.x * 8 + i) % n_vec];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            if constexpr (FP8) {
                i32x8 a = {w[u & 1][0], w[u & 1][1], w[u & 1][2], w[u & 1][3], w[2 + (u & 1)][0], w[2 + (u & 1)][1],
                           w[2 + (u & 1)][2], w[2 + (u & 1)][3]};
                const int s = 4 + 2 * ((u >> 1) & 1);
                i32x8 b = {w[s][0], w[s][1], w[s][2], w[s][3], w[s + 1][0], w[s + 1][1], w[s + 1][2], w[s + 1][3]};
                acc[u & 3] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[u & 3], 0, 0, 0, 0x7F7F7F7F, 0,
                                                                            0x7F7F7F7F);
            } else {
                acc[u & 3] = Elem<bf16_tag>::mma(w[u & 3], w[4 + ((u >> 2) & 3)], acc[u & 3]);
            }
        }
    }
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int q = 0; q < 16; ++q) r += acc[i][q];
    // keeps the loop alive; `sink` receives one float per thread of a workgroup at most
    if (r == 12345.678f) sink[threadIdx.x] = r;
}

int launch_probe_mfma(const void* operands, size_t operand_bytes, float* sink, int iters, bool fp8, hipStream_t stream) {
    const int n_vec = (int)(operand_bytes / 16);
    if (fp8)
        hipLaunchKernelGGL(fa_probe_mfma_kernel<true>, dim3(kProbeWgs), dim3(kProbeThreads), 0, stream,
                           (const i32x4*)operands, n_vec, sink, iters);
    else
        hipLaunchKernelGGL(fa_probe_mfma_kernel<false>, dim3(kProbeWgs), dim3(kProbeThreads), 0, stream,
                           (const i32x4*)operands, n_vec, sink, iters);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

double probe_mfma_flops(int iters, bool fp8) {
    const double per_mfma = fp8 ? 2.0 * 32 * 32 * 64 : 2.0 * 32 * 32 * 16;
    return (double)kProbeWgs * (kProbeThreads / 64) * (double)iters * kProbeUnroll * per_mfma;
}

}  // namespace fa
