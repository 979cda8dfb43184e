// FP8 (e4m3) forward attention for gfx950 (paper section 3.3).
//
// Same tiling as the 16-bit kernel (Algorithm 1), on v_mfma_f32_32x32x64_f8f6f4: both GEMMs
// contract 64 elements per instruction and a lane holds 32 bytes of an operand.
//   * Block quantisation: a block of S is rescaled by s_Q[i] * s_K[j], folded into the exp2
//     multiplier, so it costs nothing per element.  A V block's scale enters as an offset in
//     the exponent of P~ (the numerator's weights are p * s_V), which costs nothing either.
//   * Layout conformance: V is stored d-contiguous but must be contracted over keys.  The
//     transposing LDS read (ds_read_b64_tr_b8) hands a lane 8 consecutive keys of one column,
//     while the fp32 accumulator of S^T gives a lane-half alternating groups of 4 rows.  The
//     rows of the K operand are therefore permuted (row i of the MFMA reads key pi(i)) so
//     that each lane-half ends up owning two runs of 8 consecutive keys; P~ then goes from
//     accumulator registers to operand registers with conversions only, no cross-lane moves.
//     This is the same idea as the paper's register permutation plus matching V-row
//     permutation, rederived for the gfx950 layouts.
//   * P~ = exp2(s - m_ref + 6) where the reference maximum m_ref is raised only when a block's
//     maximum exceeds it by more than 2 (log2 units), so P~ <= 256 < 448: the bias uses more of
//     e4m3's range, both factors cancel in O / l, and L subtracts the bias again.
#include "fa_device.h"
#include "fa_launch.h"

// Measurement builds only (paper_2407_08608_amd/ablate.py compiles this file with them; the library never
// defines them).  FA_ABLATE removes one part of fa_fwd_fp8_kernel's block to see what the rest costs -- the
// results are wrong on purpose: 1 = no exponentials, 2 = no LDS reads for the second GEMM, 3 = no second GEMM,
// 4 = no softmax arithmetic (scale, exponential, row sum).  FA_PHASE_TRACE stamps the phases of 32 blocks
// of one workgroup of the eight-wave d = 128 instantiation with the shader clock.
#ifndef FA_ABLATE
#define FA_ABLATE 0
#endif
#ifdef FA_PHASE_TRACE
__device__ long long fa_phase_trace[8][32][8];
extern "C" int fa_debug_read_phase_trace(void* host) {
    return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(fa_phase_trace), sizeof(fa_phase_trace));
}
#define FA_STAMP(i) do { if (tracing) stamps[i] = __builtin_readcyclecounter(); } while (0)
#define FA_STAMP_AFTER(i, ...) do { if (tracing) { asm volatile("s_nop 0" : __VA_ARGS__); stamps[i] = __builtin_readcyclecounter(); } } while (0)
#else
#define FA_STAMP(i) do { } while (0)
#define FA_STAMP_AFTER(i, ...) do { } while (0)
#endif

namespace fa {

constexpr float kPBias = 6.0f;
constexpr float kLazyLog2 = 2.0f;

static __device__ __forceinline__ f32x16 mma_fp8(i32x8 a, i32x8 b, f32x16 c) {
    // cbsz = blgp = 0: both operands e4m3; scale exponents 127 = 1.0
    return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
}

// key held in MFMA row i of a 32-key tile
static __device__ __forceinline__ int key_of_row(int i) {
    int g = i >> 3, hb = (i >> 2) & 1, r = i & 3;
    return 16 * (g >> 1) + 8 * hb + 4 * (g & 1) + r;
}

template <int D, int BC, int NW, bool CAUSAL, bool SCALED>
__global__ void __launch_bounds__(NW * 64, D <= 128 ? 2 : 1)
fa_fwd_fp8_kernel(const uint8_t* __restrict__ q, const uint8_t* __restrict__ k, const uint8_t* __restrict__ v,
                  const float* __restrict__ q_scale, const float* __restrict__ k_scale,
                  const float* __restrict__ v_scale, uint16_t* __restrict__ o, float* __restrict__ lse, int N,
                  int n_qtiles, int total_wg, int n_sblocks, int kv_group, float scale) {
    ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int NT = NW * 64;
    constexpr int BR = NW * 32;
    constexpr int KSTR = D + 16;  // bytes per LDS row
    constexpr int VSTR = D + 32;
    constexpr int KT = BC / 32;
    constexpr int KS = D / 64;    // MFMA steps along the head dimension
    constexpr int DT = D / 32;
    constexpr int SL = BC / 64;   // MFMA steps along the keys
    constexpr int CPR = D / 16;   // 16-byte chunks per row
    constexpr int CPT = BC * CPR / NT;
    static_assert(BC % 64 == 0 && 128 % BC == 0, "key block must tile the 128-row quantisation block");
    static_assert((BC * CPR) % NT == 0, "tile must divide evenly over the workgroup");

    __shared__ __attribute__((aligned(16))) uint8_t lds_k[2][BC * KSTR];
    __shared__ __attribute__((aligned(16))) uint8_t lds_v[2][BC * VSTR];
    __shared__ __attribute__((aligned(128))) char lds_o[NW * 4096];  // output transposition, 4 KiB per wave

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    // Work items.  Non-causal: one query tile.  Causal: query tiles i and n_qtiles-1-i of a head,
    // one after the other, so that every item covers the same number of key blocks (with an odd
    // tile count the middle tile is an item of its own).
    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int n_items = CAUSAL ? (n_qtiles + 1) / 2 : n_qtiles;
    const int bh = id / n_items;
    const int item = id % n_items;
    const int n_pass = (CAUSAL && n_qtiles - 1 - item != item) ? 2 : 1;

    const size_t head_off = (size_t)bh * N * D;
    const uint8_t* qh = q + head_off;
    const int kv_bh = bh / kv_group;  // grouped-query: kv_group query heads per K/V head
    const uint8_t* kh = k + (size_t)kv_bh * N * D;
    const uint8_t* vh = v + (size_t)kv_bh * N * D;
#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    // the longer tile first; every LDS read of the previous pass was followed by a barrier
    const int qt = CAUSAL ? (pass == 0 ? n_qtiles - 1 - item : item) : item;
    const int wave_q0 = qt * BR + wave * 32;

    float sq = 1.0f;
    if constexpr (SCALED) sq = q_scale[(size_t)bh * n_sblocks + min(wave_q0 / 128, n_sblocks - 1)];
    const float sc_q = scale * kLog2e * sq;

    i32x8 qreg[KS];
    {
        int row = min(wave_q0 + col, N - 1);  // rows past N compute a copy of row N-1, never stored
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint8_t* p = qh + (size_t)row * D + ks * 64 + half * 32;
            i32x4 lo = *reinterpret_cast<const i32x4*>(p);
            i32x4 hi = *reinterpret_cast<const i32x4*>(p + 16);
            qreg[ks] = i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    }

    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    // m: running (lazily raised) maximum, in log2 units, of the real scores plus log2 of their V block's scale
    float m_run = -INFINITY, l_run = 0.f;

    int last_q = min(qt * BR + BR, N) - 1;
    int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);

    // a [BC][D] tile of a row-major head is contiguous: chunk c sits at tile offset 16*c; rows past N
    // lie outside the buffer resource and read as zero
    const __amdgpu_buffer_rsrc_t k_rsrc = make_buffer(kh, (uint32_t)N * D);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_buffer(vh, (uint32_t)N * D);
    auto load_tile = [&](__amdgpu_buffer_rsrc_t head, int key0, i32x4 (&regs)[CPT]) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) regs[i] = buffer_load_16B(head, key0 * D + (tid + i * NT) * 16);
    };
    auto store_tile = [&](uint8_t* lds, int stride, const i32x4 (&regs)[CPT]) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = tid + i * NT;
            int row = c / CPR, cc = c % CPR;
            *reinterpret_cast<i32x4*>(lds + row * stride + cc * 16) = regs[i];
        }
    };

    i32x4 kpre[CPT], vpre[CPT];
    load_tile(k_rsrc, 0, kpre);
    load_tile(v_rsrc, 0, vpre);
    store_tile(lds_k[0], KSTR, kpre);
    store_tile(lds_v[0], VSTR, vpre);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));  // Q loads complete before the loop
    __syncthreads();

    const int krow = key_of_row(col);  // key (within a 32-key tile) this lane's A row reads
    const int tr_row = (lane & 15) >> 1;
    const int tr_col = 16 * ((lane >> 4) & 1) + 8 * (lane & 1);

    for (int t = 0; t < n_blocks; ++t) {
        const int st = t & 1;
        const int key0 = t * BC;
        const bool more = (t + 1 < n_blocks);
#ifdef FA_PHASE_TRACE
        const bool tracing = D == 128 && NW == 8 && !CAUSAL && blockIdx.x == 300 && t >= 60 && t < 92;
        long long stamps[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#endif
        FA_STAMP(0);
        if (more) {
            load_tile(k_rsrc, key0 + BC, kpre);
            load_tile(v_rsrc, key0 + BC, vpre);
        }
        const bool wave_active = !CAUSAL || key0 <= wave_q0 + 31;
        if (wave_active) {
            float sk = 1.0f, sv_new = 1.0f;
            if constexpr (SCALED) {
                sk = k_scale[(size_t)kv_bh * n_sblocks + key0 / 128];
                sv_new = v_scale[(size_t)kv_bh * n_sblocks + key0 / 128];
            }
            const float sc = sc_q * sk;

            // ---- GEMM0: S^T = K_j Q_i^T (rows permuted by key_of_row)
            f32x16 sacc[KT];
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    const uint8_t* p = lds_k[st] + (kt * 32 + krow) * KSTR + ks * 64 + half * 32;
                    i32x4 lo = *reinterpret_cast<const i32x4*>(p);
                    i32x4 hi = *reinterpret_cast<const i32x4*>(p + 16);
                    i32x8 a = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    sacc[kt] = mma_fp8(a, qreg[ks], ks == 0 ? zero : sacc[kt]);
                }

            FA_STAMP_AFTER(1, "+v"(sacc[0]), "+v"(sacc[KT - 1]));  // scores done
            const bool need_mask = (key0 + BC > N) || (CAUSAL && key0 + BC - 1 > wave_q0);
            if (need_mask) {
                int qi = wave_q0 + col;
                int limit = CAUSAL ? min(qi, N - 1) : N - 1;
                // register r of lane-half `half` holds key 16 (r / 8) + 8 half + r % 8 of its 32-key tile (the
                // rows of the K operand are permuted); compile-time offsets against one opaque per-lane bound
                int bound = limit - key0 - 8 * half;
                asm volatile("" : "+v"(bound));
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kt * 32 + 16 * (r >> 3) + (r & 7) > bound) sacc[kt][r] = -INFINITY;
            }

            // ---- online softmax in log2 units of the real scores.  Independent chains for the maximum
            // and the sum: a wave gets few issue slots while its SIMD sibling streams MFMAs, and one
            // long dependent chain would turn every slot missed into a stall.
            float mxp[4] = {sacc[0][0], sacc[0][1], sacc[0][2], sacc[0][3]};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mxp[r & 3] = fmaxf(mxp[r & 3], sacc[kt][r]);
            // V block scales: O = sum_k p_k s_V[j] V^_k / sum_k p_k.  The numerator's weights are
            // 2^(s_k + log2 s_V[j]), so the block's scale is an offset in the exponent of P~ -- no work
            // per element -- and the running maximum is taken over the offset scores: P~ <= 2^(6+2) for
            // every block, and the key that raises the maximum gets P~ = 2^6 exactly.  The row sum needs
            // the weights without the offset: the block's sum divided by s_V[j], once per block.
            float lsv = 0.f;
            if constexpr (SCALED) lsv = __builtin_amdgcn_logf(sv_new);  // log2
            const float mx = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3]))) * sc + lsv;
            const bool raise = mx - m_run > kLazyLog2;
            if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                const float f = raise ? fast_exp2(m_run - mx) : 1.0f;
                m_run = raise ? mx : m_run;
                l_run *= f;
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= f;
            }
            FA_STAMP(2);  // mask, row maximum, reference
            const float mb = m_run - kPBias - lsv;
            float sc_v = sc;  // a vector-register copy: an FMA with a scalar-register operand issues at a lower rate
            asm volatile("" : "+v"(sc_v));
            float ps[4] = {0.f, 0.f, 0.f, 0.f};
            i32x8 pb[SL];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                float p[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
#if FA_ABLATE == 1
                    p[r] = __builtin_fmaf(sacc[kt][r], sc_v, -mb);
#elif FA_ABLATE == 4
                    p[r] = sacc[kt][r];
#else
                    p[r] = fast_exp2(__builtin_fmaf(sacc[kt][r], sc_v, -mb));
#endif
#if FA_ABLATE != 4
                    ps[r & 3] += p[r];
#endif
                }
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    int word = 0;
                    word = __builtin_amdgcn_cvt_pk_fp8_f32(p[4 * w], p[4 * w + 1], word, false);
                    word = __builtin_amdgcn_cvt_pk_fp8_f32(p[4 * w + 2], p[4 * w + 3], word, true);
                    pb[kt >> 1][4 * (kt & 1) + w] = word;
                }
            }
            float psum = (ps[0] + ps[1]) + (ps[2] + ps[3]);
            if constexpr (SCALED) psum *= __builtin_amdgcn_rcpf(sv_new);
            l_run += psum;

            FA_STAMP_AFTER(3, "+v"(pb[0]), "+v"(l_run));  // P~ done
            // ---- GEMM1: O^T += V_j^T P^T
            const uint8_t* vs_base = lds_v[st] + (8 * half + tr_row) * VSTR + tr_col;
#pragma unroll
            for (int sl = 0; sl < SL; ++sl)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    i32x8 a;
#if FA_ABLATE == 2
                    a = qreg[0];
                    asm volatile("" : "+v"(a));
#else
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        i32x2 w = lds_read_tr8(vs_base + (sl * 64 + 16 * u) * VSTR + dt * 32);
                        a[2 * u] = w[0];
                        a[2 * u + 1] = w[1];
                    }
#endif
#if FA_ABLATE == 3
                    asm volatile("" ::"v"(a), "v"(pb[sl]));
#else
                    oacc[dt] = mma_fp8(a, pb[sl], oacc[dt]);
#endif
                }
        }
        FA_STAMP_AFTER(4, "+v"(oacc[0]), "+v"(oacc[DT - 1]));  // products done
        if (more) {
            store_tile(lds_k[st ^ 1], KSTR, kpre);
            store_tile(lds_v[st ^ 1], VSTR, vpre);
        }
        FA_STAMP(5);  // next tiles written to LDS
        __syncthreads();
        FA_STAMP(6);  // barrier passed
#ifdef FA_PHASE_TRACE
        if (tracing && lane == 0)
            for (int i = 0; i < 7; ++i) fa_phase_trace[wave][t - 60][i] = stamps[i];
#endif
    }

    // ---- epilogue: O * s_V / l as bf16 (transposed through a wave-private LDS patch), L
    {
        char* patch = lds_o + wave * 4096;
        const int qi = wave_q0 + col;
        const float l = sum_both_halves(l_run);
        store_rows_via_lds<bf16_tag, DT>(oacc, 1.0f / l, patch, make_buffer(o + head_off, (uint32_t)N * D * 2),
                                         wave_q0, lane);
        if (qi < N && half == 0) lse[(size_t)bh * N + qi] = (m_run + log2f(l) - kPBias) * kLn2;
    }
    }  // passes of a causal pair
}

// ---------------------------------------------------------------------------------------
// Head dimension 256: four waves, one per SIMD, software-pipelined across key blocks like
// fa_fwd_d256_kernel of the 16-bit path (the paper's Algorithm 2 within one wave):
//   stage A: S(t+1)^T = K(t+1) Q^T   ||  reference maximum for S(t) (rarely a rescale of O, l),
//                                        P~(t) = exp2(...), row sums, conversion to e4m3
//   stage B: O^T += V(t)^T P~(t)^T   ||  mask and row maxima of S(t+1)
// Score tiles are produced by MfmaFp8VgprAcc into ordinary registers (O lives in the accumulation
// half of the register file), the K and V blocks travel global -> registers -> LDS one 16-byte
// chunk at a time spread over the MFMA steps, and the block scales of block t+1 are fetched a
// block ahead so that no wave waits for a scalar load.  The arithmetic is that of
// fa_fwd_fp8_kernel, step for step.
template <int D, int NW, bool CAUSAL, bool SCALED>
__global__ void __launch_bounds__(NW * 64, NW == 4 ? 1 : 2)
fa_fwd_fp8_pipe_kernel(const uint8_t* __restrict__ q, const uint8_t* __restrict__ k, const uint8_t* __restrict__ v,
                       const float* __restrict__ q_scale, const float* __restrict__ k_scale,
                       const float* __restrict__ v_scale, uint16_t* __restrict__ o, float* __restrict__ lse, int N,
                       int n_qtiles, int total_wg, int n_sblocks, int kv_group, float scale) {
    ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int BC = 64, NT = NW * 64, BR = NW * 32;
    // One wave per SIMD (d = 256, four waves): score MFMAs in inline assembly with explicit waits.  Two waves
    // per SIMD (d = 128, eight waves): at most 256 registers per lane, every MFMA result is in ordinary
    // registers anyway and the compiler's own MFMAs and hazard handling do.
    constexpr bool ONE_WAVE = NW == 4;
    constexpr int KSTR = D + 16, VSTR = D + 32;  // bytes per LDS row
    constexpr int KS = D / 64, DT = D / 32;
    constexpr int CPR = D / 16, CPT = BC * CPR / NT;  // 16-byte chunks per row, per thread and tile
    constexpr int NA = 2 * KS, NB = DT;               // MFMA steps of stage A (kt, ks) and of stage B (d-tile)
    constexpr int CH_A = NA / CPT, CH_B = NB / CPT;   // a staging chunk every so many steps
    static_assert(CPT * CH_A == NA && CPT * CH_B == NB, "chunks must spread evenly over the steps");
    static_assert(NA == 4 || NA == 8, "eight words of P~ over the steps of stage A");
    constexpr int WPS = 8 / NA;  // words of P~ (four scores each) per step of stage A

    __shared__ __attribute__((aligned(16))) uint8_t lds_k[2][BC * KSTR];
    __shared__ __attribute__((aligned(16))) uint8_t lds_v[2][BC * VSTR];
    __shared__ __attribute__((aligned(128))) char lds_o[NW * 4096];  // output transposition, 4 KiB per wave

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int n_items = CAUSAL ? (n_qtiles + 1) / 2 : n_qtiles;
    const int bh = id / n_items;
    const int item = id % n_items;
    const int n_pass = (CAUSAL && n_qtiles - 1 - item != item) ? 2 : 1;

    const size_t head_off = (size_t)bh * N * D;
    const uint8_t* qh = q + head_off;
    const int kv_bh = bh / kv_group;  // grouped-query: kv_group query heads per K/V head
    const __amdgpu_buffer_rsrc_t k_rsrc = make_buffer(k + (size_t)kv_bh * N * D, (uint32_t)N * D);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_buffer(v + (size_t)kv_bh * N * D, (uint32_t)N * D);
    const float* ksc = k_scale + (size_t)kv_bh * n_sblocks;
    const float* vsc = v_scale + (size_t)kv_bh * n_sblocks;
    const int krow = key_of_row(col);  // key (within a 32-key tile) this lane's A row reads
    const int tr_row = (lane & 15) >> 1;
    const int tr_col = 16 * ((lane >> 4) & 1) + 8 * (lane & 1);
    int unit = 0x7F7F7F7F;  // scale exponents 127 = 1.0 for both MFMA operands
    asm volatile("" : "+v"(unit));

#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    const int qt = CAUSAL ? (pass == 0 ? n_qtiles - 1 - item : item) : item;  // the longer tile first
    const int wave_q0 = qt * BR + wave * 32;
    const int limit = CAUSAL ? min(wave_q0 + col, N - 1) : N - 1;  // last key this lane's query sees

    float sq = 1.0f;
    if constexpr (SCALED) sq = q_scale[(size_t)bh * n_sblocks + min(wave_q0 / 128, n_sblocks - 1)];
    const float sc_q = scale * kLog2e * sq;

    i32x8 qreg[KS];
    {
        const int row = min(wave_q0 + col, N - 1);  // rows past N compute a copy of row N-1, never stored
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const uint8_t* p = qh + (size_t)row * D + ks * 64 + half * 32;
            i32x4 lo = *reinterpret_cast<const i32x4*>(p);
            i32x4 hi = *reinterpret_cast<const i32x4*>(p + 16);
            qreg[ks] = i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        }
    }
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    // m: running (lazily raised) maximum, in log2 units, of the real scores plus log2 of their V block's scale
    float m_run = -INFINITY, l_run = 0.f;

    const int last_q = min(qt * BR + BR, N) - 1;
    const int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);

    float mxp[4];
    auto need_mask = [&](int t) { return (t * BC + BC > N) || (CAUSAL && t * BC + BC - 1 > wave_q0); };
    auto mask_block = [&](int t, f32x16 (&s)[2]) {
        // register r of lane-half `half` holds key 16 (r / 8) + 8 half + r % 8 of its 32-key tile (the rows of
        // the K operand are permuted, see key_of_row); compile-time offsets against one opaque per-lane bound
        int bound = limit - t * BC - 8 * half;
        asm volatile("" : "+v"(bound));
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (kt * 32 + 16 * (r >> 3) + (r & 7) > bound) s[kt][r] = -INFINITY;
    };
    auto max_part = [&](f32x16 (&s)[2], int part) {  // registers 8 part .. 8 part + 7 of the 32
#pragma unroll
        for (int i = 8 * part; i < 8 * part + 8; ++i)
            mxp[i & 3] = i < 4 ? s[0][i] : fmaxf(mxp[i & 3], s[i >> 4][i & 15]);
    };
    // step u = (ks, kt) of S^T = K Q^T: the A operand is 32 bytes of a (permuted) K row
    auto k_read = [&](uint32_t k_rows, int u, i32x4& lo, i32x4& hi) {
        const uint32_t a = k_rows + ((u % 2) * 32 * KSTR + (u / 2) * 64);
        lo = lds_load_16B(a);
        hi = lds_load_16B(a + 16);
    };
    auto score_step = [&](f32x16 (&s)[2], uint32_t k_rows, i32x4 (&alo)[2], i32x4 (&ahi)[2], int u) {
        const int kt = u % 2, ks = u / 2;
        const i32x8 a = {alo[u % 2][0], alo[u % 2][1], alo[u % 2][2], alo[u % 2][3],
                         ahi[u % 2][0], ahi[u % 2][1], ahi[u % 2][2], ahi[u % 2][3]};
        if (u + 2 < NA) k_read(k_rows, u + 2, alo[u % 2], ahi[u % 2]);
        if constexpr (ONE_WAVE) {
            if (ks == 0) MfmaFp8VgprAcc::first(s[kt], a, qreg[ks], unit);
            else MfmaFp8VgprAcc::run(s[kt], a, qreg[ks], unit);
        } else {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            s[kt] = mma_fp8(a, qreg[ks], ks == 0 ? zero : s[kt]);
        }
    };
    // Scale of the 128-key block that holds key block t.  Fetched with a vector load (the index is made
    // opaque so that the compiler cannot turn it into a scalar load): scalar loads share their counter
    // with the LDS reads, and the first LDS wait after one would make the wave sit out its latency.
    auto block_scale = [&](const float* table, int t) {
        if constexpr (!SCALED) return 1.0f;
        int idx = min(t * BC / 128, n_sblocks - 1);
        asm volatile("" : "+v"(idx));
        return table[idx];
    };

    // Staging as in fa_fwd_d256_kernel, one 16-byte chunk per thread at a time spread over the MFMA
    // steps, but with a whole block of lead: the stages of this kernel are shorter than a global load,
    //   stage A of block t: write the K(t+2) chunk loaded in block t-1, load the K(t+3) chunk
    //   stage B of block t: write the V(t+1) chunk loaded in block t-1, load the V(t+2) chunk
    // (K(t+2) replaces K(t), last read in block t-1; V(t+1) replaces V(t-1), last read in block t-1.)
    i32x4 kpre[CPT], vpre[CPT];
    auto load_chunk = [&](__amdgpu_buffer_rsrc_t rsrc, int block_idx, int i) {
        return buffer_load_16B(rsrc, block_idx * BC * D + (tid + i * NT) * 16);
    };
    auto store_chunk = [&](uint8_t* lds, int stride, int i, const i32x4& x) {
        const int c = tid + i * NT;
        *reinterpret_cast<i32x4*>(lds + (c / CPR) * stride + (c % CPR) * 16) = x;
    };
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        kpre[i] = load_chunk(k_rsrc, 0, i);
        vpre[i] = load_chunk(v_rsrc, 0, i);
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i) {
        store_chunk(lds_k[0], KSTR, i, kpre[i]);
        store_chunk(lds_v[0], VSTR, i, vpre[i]);
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i) kpre[i] = load_chunk(k_rsrc, 1, i);  // K(1)
    float sk_cur = block_scale(ksc, 0), sv_cur = block_scale(vsc, 0);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {  // Q loads complete; with one wave per SIMD, Q moves to the accumulation half
        if constexpr (ONE_WAVE) asm volatile("" : "+a"(qreg[ks]));
        else asm volatile("" : "+v"(qreg[ks]));
    }
    __syncthreads();

    // ---- prologue: S(0) and its reference maximum (O and l are still zero: nothing to rescale)
    f32x16 sa[2], sb[2];
    {
        uint32_t k_rows = lds_address(lds_k[0]) + krow * KSTR + half * 32;
        asm volatile("" : "+v"(k_rows));
        i32x4 alo[2], ahi[2];
        k_read(k_rows, 0, alo[0], ahi[0]);
        k_read(k_rows, 1, alo[1], ahi[1]);
#pragma unroll
        for (int u = 0; u < NA; ++u) {
            score_step(sa, k_rows, alo, ahi, u);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < CPT; ++i) store_chunk(lds_k[1], KSTR, i, kpre[i]);
        // The loads in flight at the loop's entry are issued in the order the loop itself issues them (K
        // chunks, then V chunks): the wait counts inside the loop are compile-time numbers that must hold
        // on both paths into it, and an entry with fewer loads behind a chunk than the steady state has
        // would make every iteration wait for its newest loads.
#pragma unroll
        for (int i = 0; i < CPT; ++i) kpre[i] = load_chunk(k_rsrc, 2, i);  // K(2), written to the LDS during block 0
#pragma unroll
        for (int i = 0; i < CPT; ++i) vpre[i] = load_chunk(v_rsrc, 1, i);  // V(1), likewise
        if constexpr (ONE_WAVE) mfma_fp8_result_wait(sa[0], sa[1]);
        if (need_mask(0)) mask_block(0, sa);
#pragma unroll
        for (int part = 0; part < 4; ++part) max_part(sa, part);
        float lsv = 0.f;
        if constexpr (SCALED) lsv = __builtin_amdgcn_logf(sv_cur);  // log2
        m_run = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3]))) * (sc_q * sk_cur) + lsv;
    }
    __syncthreads();

    // ---- one key block: `cur` holds S(t), `nxt` receives S(t+1)
    auto block = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
        // the scales of block t+1, for the next call
        const float sk_next = block_scale(ksc, t + 1), sv_next = block_scale(vsc, t + 1);
        i32x8 pb;  // P~(t)^T as the B operand: 64 keys
        float ps[4] = {0.f, 0.f, 0.f, 0.f};
        float mb = 0.f, sc_v = 0.f;
        uint32_t k_rows = lds_address(lds_k[(t + 1) & 1]) + krow * KSTR + half * 32;
        uint32_t v_tr = lds_address(lds_v[t & 1]) + (8 * half + tr_row) * VSTR + tr_col;
        asm volatile("" : "+v"(k_rows), "+v"(v_tr));

        // ---- stage A
        {
            i32x4 alo[2], ahi[2];
            k_read(k_rows, 0, alo[0], ahi[0]);
            k_read(k_rows, 1, alo[1], ahi[1]);
#pragma unroll
            for (int u = 0; u < NA; ++u) {
                score_step(nxt, k_rows, alo, ahi, u);
                if (u % CH_A == 0) {
                    store_chunk(lds_k[t & 1], KSTR, u / CH_A, kpre[u / CH_A]);
                    kpre[u / CH_A] = load_chunk(k_rsrc, t + 3, u / CH_A);
                }
                if (u == 0) {
                    // Reference maximum for S(t), in log2 units of the real scores plus log2 of the V block's
                    // scale (see fa_fwd_fp8_kernel), from the row maxima taken beside the previous block's
                    // products.  The MFMAs of this stage write the score registers only, so the rare rescale
                    // of O is in order here.  (Block 0: the prologue has set the reference; no rise.)
                    float lsv = 0.f;
                    if constexpr (SCALED) lsv = __builtin_amdgcn_logf(sv_cur);
                    const float sc = sc_q * sk_cur;
                    const float mx = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3]))) * sc + lsv;
                    const bool raise = mx - m_run > kLazyLog2;
                    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                        const float f = raise ? fast_exp2(m_run - mx) : 1.0f;
                        m_run = raise ? mx : m_run;
                        l_run *= f;
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[dt][r] *= f;
                    }
                    mb = m_run - kPBias - lsv;
                    sc_v = sc;  // a vector-register copy: an FMA with a scalar-register operand issues at a lower rate
                    asm volatile("" : "+v"(sc_v));
                }
                // four scores of S(t) become one word of P~, WPS words per step
#pragma unroll
                for (int w2 = 0; w2 < WPS; ++w2) {
                    const int kt = (u * WPS + w2) / 4, w = (u * WPS + w2) % 4;
                    float p[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        p[e] = fast_exp2(__builtin_fmaf(cur[kt][4 * w + e], sc_v, -mb));
                        ps[e] += p[e];
                    }
                    int word = 0;
                    word = __builtin_amdgcn_cvt_pk_fp8_f32(p[0], p[1], word, false);
                    word = __builtin_amdgcn_cvt_pk_fp8_f32(p[2], p[3], word, true);
                    // the word must exist here: left free, the compiler sinks the exponentials (and with them
                    // the products of stage B) past the branches and the barrier below, out of this stream
                    asm volatile("" : "+v"(word), "+v"(ps[0]), "+v"(ps[1]), "+v"(ps[2]), "+v"(ps[3]));
                    pb[4 * kt + w] = word;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            float psum = (ps[0] + ps[1]) + (ps[2] + ps[3]);
            if constexpr (SCALED) psum *= __builtin_amdgcn_rcpf(sv_cur);
            l_run += psum;
        }

        // ---- stage B
        {
            auto v_read = [&](int dt, i32x2 (&w)[4]) {
#pragma unroll
                for (int x = 0; x < 4; ++x) w[x] = lds_read_tr8(v_tr + (16 * x) * VSTR + dt * 32);
            };
            i32x2 wbuf[2][4];
            v_read(0, wbuf[0]);
            v_read(1, wbuf[1]);
            const bool mask_next = need_mask(t + 1);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const i32x8 a = {wbuf[u % 2][0][0], wbuf[u % 2][0][1], wbuf[u % 2][1][0], wbuf[u % 2][1][1],
                                 wbuf[u % 2][2][0], wbuf[u % 2][2][1], wbuf[u % 2][3][0], wbuf[u % 2][3][1]};
                if (u + 2 < NB) v_read(u + 2, wbuf[u % 2]);
                oacc[u] = mma_fp8(a, pb, oacc[u]);
                // issued here, not sunk past the barrier
                if constexpr (ONE_WAVE) asm volatile("" : "+a"(oacc[u]));
                else asm volatile("" : "+v"(oacc[u]));
                if constexpr (ONE_WAVE) {
                    if (u == 0) mfma_fp8_result_wait(nxt[0], nxt[1]);  // written by MFMAs the hazard checker cannot see
                }
                if (u == 1 && mask_next) mask_block(t + 1, nxt);
                if constexpr (NB == 8) {
                    if (u >= 2 && u < 6) max_part(nxt, u - 2);
                } else {
                    if (u >= 2) {
                        max_part(nxt, 2 * (u - 2));
                        max_part(nxt, 2 * (u - 2) + 1);
                    }
                }
                if (u % CH_B == 0) {
                    store_chunk(lds_v[(t + 1) & 1], VSTR, u / CH_B, vpre[u / CH_B]);
                    vpre[u / CH_B] = load_chunk(v_rsrc, t + 2, u / CH_B);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        sk_cur = sk_next;
        sv_cur = sv_next;
        lds_barrier();  // the chunk loads of this block stay in flight
    };

    for (int t = 0; t < n_blocks; t += 2) {
        block(t, sa, sb);
        if (t + 1 < n_blocks) block(t + 1, sb, sa);
    }

    // ---- epilogue: O * s_V / l as bf16 (transposed through a wave-private LDS patch), L
    {
        char* patch = lds_o + wave * 4096;
        const int qi = wave_q0 + col;
        const float l = sum_both_halves(l_run);
        store_rows_via_lds<bf16_tag, DT>(oacc, 1.0f / l, patch, make_buffer(o + head_off, (uint32_t)N * D * 2),
                                         wave_q0, lane);
        if (qi < N && half == 0) lse[(size_t)bh * N + qi] = (m_run + log2f(l) - kPBias) * kLn2;
    }
    }  // passes of a causal pair
}

template <int D, int NW>
static int launch_fp8_pipe(const void* q8, const void* k8, const void* v8, const float* qs, const float* ks,
                           const float* vs, void* o, float* lse, int B, int H, int H_kv, int N, float scale,
                           int causal, hipStream_t stream) {
    constexpr int BR = NW * 32;
    int n_qtiles = (N + BR - 1) / BR;
    int n_sblocks = (N + 127) / 128;
    long total = (long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);  // causal: tiles are paired up
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(NW * 64);
    auto qp = static_cast<const uint8_t*>(q8);
    auto kp = static_cast<const uint8_t*>(k8);
    auto vp = static_cast<const uint8_t*>(v8);
    auto op = static_cast<uint16_t*>(o);
    const bool scaled = qs != nullptr;
#define FA_LAUNCH_FP8_D256(C, S)                                                                               \
    hipLaunchKernelGGL((fa_fwd_fp8_pipe_kernel<D, NW, C, S>), grid, block, 0, stream, qp, kp, vp, qs, ks, vs, op, lse, \
                       N, n_qtiles, (int)total, n_sblocks, H / H_kv, scale)
    if (causal) {
        if (scaled) FA_LAUNCH_FP8_D256(true, true); else FA_LAUNCH_FP8_D256(true, false);
    } else {
        if (scaled) FA_LAUNCH_FP8_D256(false, true); else FA_LAUNCH_FP8_D256(false, false);
    }
#undef FA_LAUNCH_FP8_D256
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

template <int D, int BC, int NW>
static int launch_fp8(const void* q8, const void* k8, const void* v8, const float* qs, const float* ks,
                      const float* vs, void* o, float* lse, int B, int H, int H_kv, int N, float scale, int causal,
                      hipStream_t stream) {
    constexpr int BR = NW * 32;
    int n_qtiles = (N + BR - 1) / BR;
    int n_sblocks = (N + 127) / 128;
    long total = (long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);  // causal: tiles are paired up
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(NW * 64);
    auto qp = static_cast<const uint8_t*>(q8);
    auto kp = static_cast<const uint8_t*>(k8);
    auto vp = static_cast<const uint8_t*>(v8);
    auto op = static_cast<uint16_t*>(o);
    const bool scaled = qs != nullptr;
#define FA_LAUNCH_FP8(C, S)                                                                                       \
    hipLaunchKernelGGL((fa_fwd_fp8_kernel<D, BC, NW, C, S>), grid, block, 0, stream, qp, kp, vp, qs, ks, vs, op, \
                       lse, N, n_qtiles, (int)total, n_sblocks, H / H_kv, scale)
    if (causal) {
        if (scaled) FA_LAUNCH_FP8(true, true); else FA_LAUNCH_FP8(true, false);
    } else {
        if (scaled) FA_LAUNCH_FP8(false, true); else FA_LAUNCH_FP8(false, false);
    }
#undef FA_LAUNCH_FP8
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

enum class FwdFp8 { kTile4, kTile8, kPipe256, kNone };
static FwdFp8 choose_fp8(int d, int N, int causal) {
    // Short problems keep the 128-row tile of four waves (more workgroups, less waste on the diagonal); the
    // crossovers were measured on block-scaled inputs at 16k tokens per launch.
    switch (d) {
        case 64: return (causal || N <= 3072) ? FwdFp8::kTile4 : FwdFp8::kTile8;
        // (fa_fwd_fp8_pipe_kernel<128, 8>, two waves per SIMD, is correct and measured 5 % slower than the 8-wave tile)
        case 128: return N <= (causal ? 1280 : 704) ? FwdFp8::kTile4 : FwdFp8::kTile8;
        case 256: return FwdFp8::kPipe256;
        default: return FwdFp8::kNone;
    }
}

int launch_fwd_fp8(const void* q8, const void* k8, const void* v8, const float* q_scale, const float* k_scale,
                   const float* v_scale, void* o, float* lse, int B, int H, int H_kv, int N, int d, float scale, int causal,
                   hipStream_t stream) {
#define FA_FP8_ARGS q8, k8, v8, q_scale, k_scale, v_scale, o, lse, B, H, H_kv, N, scale, causal, stream
    switch (choose_fp8(d, N, causal)) {
        case FwdFp8::kTile4:
            if (d == 64) return launch_fp8<64, 64, 4>(FA_FP8_ARGS);
            return launch_fp8<128, 64, 4>(FA_FP8_ARGS);
        case FwdFp8::kTile8:
            if (d == 64) return launch_fp8<64, 128, 8>(FA_FP8_ARGS);
            return launch_fp8<128, 128, 8>(FA_FP8_ARGS);
        case FwdFp8::kPipe256: return launch_fp8_pipe<256, 4>(FA_FP8_ARGS);
        default: return FA_ERR_UNSUPPORTED;
    }
#undef FA_FP8_ARGS
}

// The name a profiler shows for the kernel launch_fwd_fp8 picks (block-scaled instantiation).
const char* fwd_fp8_kernel_name(int N, int d, int causal) {
    static const char* const names[2][5] = {
        {"fa_fwd_fp8_kernel<64, 64, 4, false, true>", "fa_fwd_fp8_kernel<128, 64, 4, false, true>",
         "fa_fwd_fp8_kernel<64, 128, 8, false, true>", "fa_fwd_fp8_kernel<128, 128, 8, false, true>",
         "fa_fwd_fp8_pipe_kernel<256, 4, false, true>"},
        {"fa_fwd_fp8_kernel<64, 64, 4, true, true>", "fa_fwd_fp8_kernel<128, 64, 4, true, true>",
         "fa_fwd_fp8_kernel<64, 128, 8, true, true>", "fa_fwd_fp8_kernel<128, 128, 8, true, true>",
         "fa_fwd_fp8_pipe_kernel<256, 4, true, true>"}};
    int idx;
    switch (choose_fp8(d, N, causal)) {
        case FwdFp8::kTile4: idx = d == 64 ? 0 : 1; break;
        case FwdFp8::kTile8: idx = d == 64 ? 2 : 3; break;
        case FwdFp8::kPipe256: idx = 4; break;
        default: return nullptr;
    }
    return names[causal ? 1 : 0][idx];
}

}  // namespace fa

FA_CLOCK_SPAN_READER(fa_debug_clock_span_fwd_fp8)
