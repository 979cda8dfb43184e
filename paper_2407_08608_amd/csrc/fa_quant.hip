// FP8 pre-pass (paper section 3.3): optional incoherent processing  y = (x * s) H_d / sqrt(d)
// followed by block quantisation to e4m3 with one fp32 scale per 128 rows of a head.
//
// HBM-bound: every element is read once (2 or 4 bytes) and written once (1 byte).  One
// workgroup owns one 128-row block; d / 16 lanes (at least four) share a row, each holding its
// part of the row as 8-element chunks interleaved across those lanes, so that global loads
// (16 bytes per lane) and stores (8 bytes) are coalesced and a lane holds 32 values of the block
// whatever the head dimension.  The Hadamard butterflies run in the order of the element index
// bits (strides 1, 2, ..., d/2): strides 1-4 inside a chunk, strides 8-16 between neighbouring
// lanes with DPP quad permutes, strides 32-64 (eight or sixteen lanes per row) with ds_swizzle lane
// exchanges, the remaining strides across the lane's chunks.  All arithmetic that decides a code is
// fp32: add/sub butterflies, one multiply by float(1/sqrt(d)), one multiply by 448/amax, clamp,
// round-to-nearest-even conversion.
#include "fa_device.h"
#include "fa_launch.h"

namespace fa {

constexpr int kBlockRows = 128;
constexpr float kE4m3Max = 448.0f;

template <int CTRL>
static __device__ __forceinline__ float quad_perm(float x) {
    int v = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true);
    return __builtin_bit_cast(float, v);
}

template <int IN_DTYPE>
static __device__ __forceinline__ void load_chunk(const void* base, size_t elem_off, float (&out)[8]) {
    if constexpr (IN_DTYPE == FA_F32) {
        const float* p = static_cast<const float*>(base) + elem_off;
        f32x4 a = *reinterpret_cast<const f32x4*>(p);
        f32x4 b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            out[t] = a[t];
            out[4 + t] = b[t];
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(base) + elem_off;
        i32x4 w = *reinterpret_cast<const i32x4*>(p);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t u = (uint32_t)w[t];
            if constexpr (IN_DTYPE == FA_BF16) {
                out[2 * t] = Elem<bf16_tag>::to_float((uint16_t)(u & 0xFFFF));
                out[2 * t + 1] = Elem<bf16_tag>::to_float((uint16_t)(u >> 16));
            } else {
                out[2 * t] = Elem<f16_tag>::to_float((uint16_t)(u & 0xFFFF));
                out[2 * t + 1] = Elem<f16_tag>::to_float((uint16_t)(u >> 16));
            }
        }
    }
}

// MODE 0: per-block scales.  MODE 1: only fold the block's amax into *amax_bits (atomic max on
// the bit pattern of a non-negative float).  MODE 2: quantise with the scale taken from
// *amax_bits, leave `scales` alone.
// Lanes per row: d / 16 (at least 4), so that a lane holds 32 values of the 128-row block whatever
// the head dimension and six waves fit a SIMD: the kernel is bound by memory latency otherwise.
constexpr int quant_lanes_per_row(int d) { return d >= 64 ? (d / 16 < 4 ? 4 : d / 16) : 4; }

template <int D, int IN_DTYPE, int MODE, bool HADAMARD>
__global__ void __launch_bounds__(64 * quant_lanes_per_row(D))
fa_quant_kernel(const void* __restrict__ x, uint8_t* __restrict__ x8, float* __restrict__ scales,
                const signed char* __restrict__ signs, unsigned* amax_bits, int N, int n_blocks) {
    constexpr int LPR = quant_lanes_per_row(D);
    constexpr int CH = D / (8 * LPR);        // 8-element chunks per lane
    constexpr int PASSES = kBlockRows / 64;  // 64 rows per pass over the workgroup
    const int tid = threadIdx.x;
    const int p = tid & (LPR - 1);    // lane within the row's group
    const int row_in_pass = tid / LPR;
    const int bh = blockIdx.x / n_blocks, blk = blockIdx.x % n_blocks;
    const size_t head_off = (size_t)bh * N * D;
    const float inv_sqrt_d = (float)(1.0 / __builtin_sqrt((double)D));

    float sg[CH][8];
    if constexpr (HADAMARD) {
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int t = 0; t < 8; ++t) sg[c][t] = (float)signs[8 * (p + LPR * c) + t];
    }

    float y[PASSES][CH][8];
    float amax = 0.f;
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int row = blk * kBlockRows + ps * 64 + row_in_pass;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            if (row < N) {
                load_chunk<IN_DTYPE>(x, head_off + (size_t)row * D + 8 * (p + LPR * c), y[ps][c]);
            } else {
#pragma unroll
                for (int t = 0; t < 8; ++t) y[ps][c][t] = 0.f;
            }
        }
        if constexpr (HADAMARD) {
            // element index e = t + 8*p + 8*LPR*c
#pragma unroll
            for (int c = 0; c < CH; ++c) {
#pragma unroll
                for (int t = 0; t < 8; ++t) y[ps][c][t] *= sg[c][t];
#pragma unroll
                for (int h = 1; h < 8; h <<= 1)  // strides 1, 2, 4
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if ((t & h) == 0) {
                            float a = y[ps][c][t], b = y[ps][c][t + h];
                            y[ps][c][t] = a + b;
                            y[ps][c][t + h] = a - b;
                        }
            }
            // strides 8 and 16: partner lane p^1, then p^2; low lane gets a+b, high lane a-b
            const float s1 = (p & 1) ? -1.f : 1.f, s2 = (p & 2) ? -1.f : 1.f;
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    float v = y[ps][c][t];
                    v = __builtin_fmaf(v, s1, quad_perm<0xB1>(v));  // lanes (1,0,3,2)
                    v = __builtin_fmaf(v, s2, quad_perm<0x4E>(v));  // lanes (2,3,0,1)
                    // strides 32 and 64: partner lanes p^4, p^8 (swizzle within 32 lanes: and 0x1f, or 0, xor)
                    if constexpr (LPR >= 8) {
                        const float s3 = (p & 4) ? -1.f : 1.f;
                        const float other = __builtin_bit_cast(
                            float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (4 << 10) | 0x1f));
                        v = __builtin_fmaf(v, s3, other);
                    }
                    if constexpr (LPR >= 16) {
                        const float s4 = (p & 8) ? -1.f : 1.f;
                        const float other = __builtin_bit_cast(
                            float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), (8 << 10) | 0x1f));
                        v = __builtin_fmaf(v, s4, other);
                    }
                    y[ps][c][t] = v;
                }
#pragma unroll
            for (int h = 1; h < CH; h <<= 1)  // strides 8 LPR h: 32, 64, 128 (64, 128 with eight lanes per row)
#pragma unroll
                for (int c = 0; c < CH; ++c)
                    if ((c & h) == 0)
#pragma unroll
                        for (int t = 0; t < 8; ++t) {
                            float a = y[ps][c][t], b = y[ps][c + h][t];
                            y[ps][c][t] = a + b;
                            y[ps][c + h][t] = a - b;
                        }
#pragma unroll
            for (int c = 0; c < CH; ++c)
#pragma unroll
                for (int t = 0; t < 8; ++t) y[ps][c][t] *= inv_sqrt_d;
        }
#pragma unroll
        for (int c = 0; c < CH; ++c)
#pragma unroll
            for (int t = 0; t < 8; ++t) amax = fmaxf(amax, fabsf(y[ps][c][t]));
    }

    // block amax
    static_assert(LPR <= 16, "the lane exchanges above cover up to sixteen lanes per row");
    __shared__ float red[LPR];  // one slot per wave
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    if ((tid & 63) == 0) red[tid >> 6] = amax;
    __syncthreads();
    amax = red[0];
#pragma unroll
    for (int w = 1; w < LPR; ++w) amax = fmaxf(amax, red[w]);

    if constexpr (MODE == 1) {
        if (tid == 0) atomicMax(amax_bits, __builtin_bit_cast(unsigned, amax));
        return;
    }
    if constexpr (MODE == 2) amax = __builtin_bit_cast(float, *amax_bits);

    float scale = 1.0f, inv = 1.0f;
    if (amax != 0.f) {
        scale = amax / kE4m3Max;
        inv = kE4m3Max / amax;
    }
    if (MODE == 0 && tid == 0) scales[(size_t)bh * n_blocks + blk] = scale;

#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
        const int row = blk * kBlockRows + ps * 64 + row_in_pass;
        if (row >= N) continue;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            float z[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) z[t] = fminf(fmaxf(y[ps][c][t] * inv, -kE4m3Max), kE4m3Max);
            int w0 = 0, w1 = 0;
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(z[0], z[1], w0, false);
            w0 = __builtin_amdgcn_cvt_pk_fp8_f32(z[2], z[3], w0, true);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(z[4], z[5], w1, false);
            w1 = __builtin_amdgcn_cvt_pk_fp8_f32(z[6], z[7], w1, true);
            i32x2 w = {w0, w1};
            *reinterpret_cast<i32x2*>(x8 + head_off + (size_t)row * D + 8 * (p + LPR * c)) = w;
        }
    }
}

__global__ void fa_zero_word_kernel(unsigned* p) { *p = 0u; }

// one workgroup: read the tensor-wide amax (stored as bits in slot 0), then fill every slot
__global__ void __launch_bounds__(256) fa_fill_scales_kernel(float* scales, long n) {
    float amax = __builtin_bit_cast(float, *reinterpret_cast<unsigned*>(scales));
    __syncthreads();  // every thread has read slot 0 before anyone overwrites it
    float scale = amax != 0.f ? amax / kE4m3Max : 1.0f;
    for (long i = threadIdx.x; i < n; i += 256) scales[i] = scale;
}

template <int D, int IN_DTYPE, bool HADAMARD>
static int launch_quant(const void* x, void* x8, float* scales, int B, int H, int N, const signed char* signs,
                        int per_tensor, hipStream_t stream) {
    int n_blocks = (N + kBlockRows - 1) / kBlockRows;
    long total = (long)B * H * n_blocks;
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(64 * quant_lanes_per_row(D));
    auto out = static_cast<uint8_t*>(x8);
    unsigned* slot0 = reinterpret_cast<unsigned*>(scales);
    if (!per_tensor) {
        hipLaunchKernelGGL((fa_quant_kernel<D, IN_DTYPE, 0, HADAMARD>), grid, block, 0, stream, x, out, scales, signs,
                           slot0, N, n_blocks);
    } else {
        hipLaunchKernelGGL(fa_zero_word_kernel, dim3(1), dim3(1), 0, stream, slot0);
        if (hipGetLastError() != hipSuccess) return FA_ERR_LAUNCH;
        hipLaunchKernelGGL((fa_quant_kernel<D, IN_DTYPE, 1, HADAMARD>), grid, block, 0, stream, x, out, scales, signs,
                           slot0, N, n_blocks);
        if (hipGetLastError() != hipSuccess) return FA_ERR_LAUNCH;
        hipLaunchKernelGGL((fa_quant_kernel<D, IN_DTYPE, 2, HADAMARD>), grid, block, 0, stream, x, out, scales, signs,
                           slot0, N, n_blocks);
        if (hipGetLastError() != hipSuccess) return FA_ERR_LAUNCH;
        hipLaunchKernelGGL(fa_fill_scales_kernel, dim3(1), dim3(256), 0, stream, scales, total);
    }
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

template <int D, int IN_DTYPE>
static int launch_quant_h(const void* x, void* x8, float* scales, int B, int H, int N, const signed char* signs,
                          int per_tensor, hipStream_t stream) {
    return signs ? launch_quant<D, IN_DTYPE, true>(x, x8, scales, B, H, N, signs, per_tensor, stream)
                 : launch_quant<D, IN_DTYPE, false>(x, x8, scales, B, H, N, signs, per_tensor, stream);
}

template <int IN_DTYPE>
static int launch_quant_d(const void* x, void* x8, float* scales, int B, int H, int N, int d,
                          const signed char* signs, int per_tensor, hipStream_t stream) {
    switch (d) {
        case 64: return launch_quant_h<64, IN_DTYPE>(x, x8, scales, B, H, N, signs, per_tensor, stream);
        case 128: return launch_quant_h<128, IN_DTYPE>(x, x8, scales, B, H, N, signs, per_tensor, stream);
        case 256: return launch_quant_h<256, IN_DTYPE>(x, x8, scales, B, H, N, signs, per_tensor, stream);
        default: return FA_ERR_UNSUPPORTED;
    }
}

int launch_quant_hadamard(const void* x, int in_dtype, void* x8, float* scales, int B, int H, int N, int d,
                          const signed char* signs, int per_tensor, hipStream_t stream) {
    switch (in_dtype) {
        case FA_F32: return launch_quant_d<FA_F32>(x, x8, scales, B, H, N, d, signs, per_tensor, stream);
        case FA_BF16: return launch_quant_d<FA_BF16>(x, x8, scales, B, H, N, d, signs, per_tensor, stream);
        case FA_F16: return launch_quant_d<FA_F16>(x, x8, scales, B, H, N, d, signs, per_tensor, stream);
        default: return FA_ERR_UNSUPPORTED;
    }
}

}  // namespace fa
