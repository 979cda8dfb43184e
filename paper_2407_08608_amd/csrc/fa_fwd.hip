// Forward attention kernels for gfx950: 16-bit (bf16 / fp16) MFMA path and the fp32 path.
//
// One workgroup owns a tile of BR = NW * 32 * RQ query rows of one (batch, head) and walks
// the key/value blocks of that head (paper Algorithm 1: T_r query tiles on the grid, T_c
// key blocks in the inner loop).  Per block: S^T = K_j Q_i^T on MFMA, online softmax with
// running row maximum m and row sum l, O^T += V_j^T P^T on MFMA, O rescaled by
// exp(m_old - m_new); epilogue O / l and L = m + log l.  K_j and V_j are staged through a
// double-buffered LDS ring that the next block's global loads fill while the current block
// is being computed (the role the producer warpgroup plays in the paper).
#include <type_traits>

#include "fa_device.h"
#include "fa_launch.h"

// Measurement builds only (paper_2407_08608_amd/ablate.py compiles this file with it; the library never defines
// it): FA_ABLATE_PP removes one part of fa_fwd_pingpong_kernel's block to see what the rest costs -- results
// wrong on purpose: 1 = no exponentials, 2 = no LDS reads of V operands, 3 = no LDS reads of K operands,
// 4 = no softmax arithmetic at all (P~ = packed scores).
#ifndef FA_ABLATE_PP
#define FA_ABLATE_PP 0
#endif

namespace fa {

constexpr float kLazyLog2 = 8.0f;
// fa_fwd_pingpong_kernel: a block whose per-lane sum of P~ exceeds this moves the row's reference (2^14:
// every P~ of a block that stays below it fits fp16 with room to spare)
constexpr float kRaiseAbove = 16384.0f;

template <int D, int BC, int NT>
struct TileCopy {
    static constexpr int kChunksPerRow = D / 8;  // 16-byte chunks of 8 16-bit elements
    static constexpr int kChunks = BC * kChunksPerRow;
    static constexpr int kPerThread = kChunks / NT;
    static_assert(kChunks % NT == 0, "tile must divide evenly over the workgroup");

    // A [BC][D] tile of a row-major [N][D] head is one contiguous run of bytes, so chunk c of the
    // tile sits at tile_byte_off + 16*c: no per-row address arithmetic.  Rows past N fall outside
    // the buffer resource and read as zero (their scores are masked anyway).
    static __device__ __forceinline__ void from_global(__amdgpu_buffer_rsrc_t head, int tile_byte_off, int tid,
                                                       i32x4 (&regs)[kPerThread]) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i)
            regs[i] = buffer_load_16B(head, tile_byte_off + (tid + i * NT) * 16);
    }
    template <int STRIDE>
    static __device__ __forceinline__ void to_lds(uint16_t* lds, int tid, const i32x4 (&regs)[kPerThread]) {
#pragma unroll
        for (int i = 0; i < kPerThread; ++i) {
            int c = tid + i * NT;
            int row = c / kChunksPerRow, col = c % kChunksPerRow;
            *reinterpret_cast<i32x4*>(lds + row * STRIDE + col * 8) = regs[i];
        }
    }
};

template <typename Tag, int D, int BC, int NW, int RQ, int PD, bool CAUSAL>
// (the second launch bound is waves per SIMD: two eight-wave workgroups of the d = 64 kernel share a CU)
__global__ void __launch_bounds__(NW * 64, (D == 64 && NW == 8) ? 4 : (RQ == 1 && D <= 128) ? 2 : 1)
fa_fwd_16bit_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                    const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse,
                    int N, int n_qtiles, int total_wg, int kv_group, float scale) {
    [[maybe_unused]] ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int NT = NW * 64;
    constexpr int BR = NW * 32 * RQ;
    constexpr int KSTR = D + 8;   // +16 B per row: 128-bit row reads hit distinct banks
    constexpr int VSTR = D + 32;  // +64 B per row: the 4-row transposing reads hit distinct banks
    constexpr int KT = BC / 32;   // 32-key score tiles per block
    constexpr int KS = D / 16;    // MFMA steps along the head dimension
    constexpr int DT = D / 32;    // 32-column output tiles
    constexpr int SL = BC / 16;   // 16-key MFMA steps along the keys
    using E = Elem<Tag>;
    using Copy = TileCopy<D, BC, NT>;

    __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][BC * KSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][BC * VSTR];

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
    const size_t kv_off = (size_t)(bh / kv_group) * N * D;  // grouped-query: kv_group query heads per K/V head
    const uint16_t* qh = q + head_off;
    const uint16_t* kh = k + kv_off;
    const uint16_t* vh = v + kv_off;

    const float sc = scale * kLog2e;  // exp(scale*s - scale*m) = exp2(sc*s - sc*m)
    float sc_v = sc;  // a vector-register copy: an FMA with a scalar-register operand issues at a lower rate
    asm volatile("" : "+v"(sc_v));

#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    // the longer tile first; every LDS read of the previous pass was followed by a barrier
    const int qt = CAUSAL ? (pass == 0 ? n_qtiles - 1 - item : item) : item;
    const int wave_q0 = qt * BR + wave * (32 * RQ);

    // Q_i^T as the B operand, resident in registers for the whole loop
    static_assert(RQ == 1 && PD == 0, "one 32-row slab per wave, operand reads scheduled by the compiler");
    i32x4 qreg[KS];
    {
        int row = min(wave_q0 + col, N - 1);  // rows past N compute a copy of row N-1, never stored
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qreg[ks] = *reinterpret_cast<const i32x4*>(qh + (size_t)row * D + ks * 16 + half * 8);
    }

    f32x16 oacc[DT];
    float m_run = 0.f, l_run = 0.f;  // reference (log2 units of the scaled scores; set by block 0) and row sum of P~
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;

    // key blocks this workgroup must visit
    int last_q = min(qt * BR + BR, N) - 1;
    int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);

    i32x4 kpre[Copy::kPerThread], vpre[Copy::kPerThread];
    const __amdgpu_buffer_rsrc_t k_rsrc = make_buffer(kh, (uint32_t)N * D * 2);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_buffer(vh, (uint32_t)N * D * 2);
    Copy::from_global(k_rsrc, 0, tid, kpre);
    Copy::from_global(v_rsrc, 0, tid, vpre);
    Copy::template to_lds<KSTR>(lds_k[0], tid, kpre);
    Copy::template to_lds<VSTR>(lds_v[0], tid, vpre);
    // Pin the Q loads' completion here.  Left to itself the compiler sinks them to the loop
    // entry, and the vmcnt waits it then needs at their first use sit inside the loop body,
    // where on every later iteration they would wait for the K/V prefetch just issued.
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));
    __syncthreads();

    // transposing V read: lane -> (row within a 4-key group, 4-column chunk) of its 16-lane group
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    for (int t = 0; t < n_blocks; ++t) {
        const int st = t & 1;
        const int key0 = t * BC;
        const bool more = (t + 1 < n_blocks);
        if (more) {
            Copy::from_global(k_rsrc, (key0 + BC) * D * 2, tid, kpre);
            Copy::from_global(v_rsrc, (key0 + BC) * D * 2, tid, vpre);
        }

        // a wave whose queries all precede this block has nothing to add (causal)
        const bool wave_active = !CAUSAL || key0 <= wave_q0 + 32 * RQ - 1;
        if (wave_active) {
            // ---- GEMM0: S^T = K_j Q_i^T, then the mask: keys past N, and keys after the query when causal
            f32x16 sacc[KT];
            const bool need_mask = (key0 + BC > N) || (CAUSAL && key0 + BC - 1 > wave_q0);
            auto scores = [&]() __attribute__((always_inline)) {
                const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                const uint16_t* ks_base = lds_k[st] + col * KSTR + half * 8;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt) {
                        i32x4 a = *reinterpret_cast<const i32x4*>(ks_base + kt * 32 * KSTR + ks * 16);
                        sacc[kt] = E::mma(a, qreg[ks], ks == 0 ? zero : sacc[kt]);
                    }
                if (need_mask) {
                    const int qi = wave_q0 + col;
                    const int limit = CAUSAL ? min(qi, N - 1) : N - 1;  // last visible key
                    // compile-time key offsets against one opaque per-lane bound: a compare and a select per
                    // score, no index arithmetic
                    int bound = limit - key0 - 4 * half;
                    asm volatile("" : "+v"(bound));
#pragma unroll
                    for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            if (kt * 32 + 8 * (r >> 2) + (r & 3) > bound) sacc[kt][r] = -INFINITY;
                }
            };
            // The row's reference m (log2 units of the scaled scores) becomes the maximum of the block in
            // `sacc` for the lanes that ask for it; O and l follow.
            auto move_reference = [&](bool wanted, auto first_block) __attribute__((always_inline)) {
                float mxp[4] = {sacc[0][0], sacc[0][1], sacc[0][2], sacc[0][3]};
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) mxp[r & 3] = fmaxf(mxp[r & 3], sacc[kt][r]);
                const float m_new = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3]))) * sc;
                if constexpr (decltype(first_block)::value) {  // O and l are still zero: only m changes
                    m_run = m_new;
                } else {
                    const float corr = wanted ? fast_exp2(m_run - m_new) : 1.0f;
                    m_run = wanted ? m_new : m_run;
                    l_run *= corr;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[dt][r] *= corr;
                }
            };
            // P~ = exp2(s c - m) packed as the operand for GEMM1; returns this lane's part of the row sum
            i32x4 pb[SL];
            auto probabilities = [&]() __attribute__((always_inline)) {
                float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    float p[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        p[r] = fast_exp2(__builtin_fmaf(sacc[kt][r], sc_v, -m_run));
                        ps[r & 3] += p[r];
                    }
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        i32x4 w;
#pragma unroll
                        for (int i = 0; i < 4; ++i) w[i] = E::pack2(p[8 * s2 + 2 * i], p[8 * s2 + 2 * i + 1]);
                        pb[2 * kt + s2] = w;
                    }
                }
                return (ps[0] + ps[1]) + (ps[2] + ps[3]);
            };

            // ---- online softmax (Algorithm 1: m, P~, l) without a row maximum per block.  The reference m
            // is block 0's true row maximum and afterwards moves only when a block's row sum of P~ --
            // computed anyway -- exceeds kRaiseAbove: below that every P~ of the block is below it too (also
            // as a 16-bit value of the fp16 path), the reference cancels in O / l, and L = m + log2 l
            // either way.  A block that does exceed it (scores that rose by more than 14 in log2 units
            // since the reference was set: rare) is computed again from the K tile, which is still in
            // LDS, with its own maximum as the new reference.
            scores();
            if (t == 0) move_reference(true, std::true_type{});
            float blk = probabilities();
            const bool over = max_both_halves(blk) > kRaiseAbove;
            if (__builtin_amdgcn_ballot_w64(over) != 0) {
                scores();
                move_reference(over, std::false_type{});
                blk = probabilities();
            }
            l_run += blk;

            // ---- GEMM1: O^T += V_j^T P^T
            const uint16_t* vs_base = lds_v[st] + (4 * half + tr_row) * VSTR + tr_col;
#pragma unroll
            for (int sl = 0; sl < SL; ++sl)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const uint16_t* p0 = vs_base + (sl * 16) * VSTR + dt * 32;
                    i32x2 lo = lds_read_tr16(p0);
                    i32x2 hi = lds_read_tr16(p0 + 8 * VSTR);
                    i32x4 a = {lo[0], lo[1], hi[0], hi[1]};
                    oacc[dt] = E::mma(a, pb[sl], oacc[dt]);
                }
        }

        if (more) {
            Copy::template to_lds<KSTR>(lds_k[st ^ 1], tid, kpre);
            Copy::template to_lds<VSTR>(lds_v[st ^ 1], tid, vpre);
        }
        __syncthreads();
    }

    // ---- epilogue: O / l, L = m + log l.  Every LDS read of the loop was followed by a barrier,
    // so the K and V buffers are free: each wave takes 4 KiB of them to transpose its output tile.
    {
        char* patch = (wave < 4 ? reinterpret_cast<char*>(&lds_k[0][0]) : reinterpret_cast<char*>(&lds_v[0][0])) +
                      (wave & 3) * 4096;
        static_assert(sizeof(lds_k) >= 4 * 4096 && sizeof(lds_v) >= 4 * 4096, "patches must fit");
        const int qi = wave_q0 + col;
        const float l = sum_both_halves(l_run);
        store_rows_via_lds<Tag, DT>(oacc, 1.0f / l, patch, make_buffer(o + head_off, (uint32_t)N * D * 2), wave_q0,
                                    lane);
        if (qi < N && half == 0) lse[(size_t)bh * N + qi] = (m_run + log2f(l)) * kLn2;
    }
    if (pass + 1 < n_pass) __syncthreads();  // the next pass's first tile overwrites the patches
    }  // passes of a causal pair
}

// ---------------------------------------------------------------------------------------
// Head dimension 256: four waves, one per SIMD.
//
// The output accumulator of 32 query rows (128 registers per lane) and the 64 registers of Q_i
// leave room for one wave per SIMD, so nothing but the wave's own instruction stream can keep
// the matrix pipe busy while the exponentials run.  The loop is therefore software-pipelined
// across key blocks the way the paper's Algorithm 2 (section 3.2) pipelines within a warpgroup:
// the scores of block t+1 are produced while the exponentials of block t run,
//   stage A: S(t+1)^T = K(t+1) Q^T     ||  reference maximum for S(t) (raised lazily; rarely a rescale
//                                          of O and l), P~(t) = exp2(S(t) - m), row sums
//   stage B: O^T += V(t)^T P~(t)^T     ||  mask and row maxima of S(t+1)
// so both score tiles are live at once (the paper's extra S_next registers), K runs one block
// ahead of V through the LDS buffers, and the only rescale of O sits at the head of stage A,
// whose MFMAs do not touch O.  O and Q live in the accumulation half of the register file, which MFMA
// alone can address; the score tiles are produced by MfmaVgprAcc into ordinary registers, where
// the softmax reads them without a copy per score.  Every step ends in a full scheduling
// barrier, so the interleaving written here is what runs, and LDS operand reads lead their
// MFMAs by KP steps.  The block after the last one is computed like any other and comes out
// fully masked (32 MFMAs per tile that add nothing).
template <typename Tag, bool CAUSAL>
__global__ void __launch_bounds__(256, 1)
fa_fwd_d256_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                   uint16_t* __restrict__ o, float* __restrict__ lse, int N, int n_qtiles, int total_wg,
                   int kv_group, float scale) {
    [[maybe_unused]] ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int D = 256, BC = 64, NT = 256, BR = 128;
    constexpr int KSTR = D + 8;   // +16 B per row: 128-bit row reads hit distinct banks
    constexpr int VSTR = D + 32;  // +64 B per row: the 4-row transposing reads hit distinct banks
    constexpr int KS = D / 16, DT = D / 32, KP = 4;
    using E = Elem<Tag>;
    using Copy = TileCopy<D, BC, NT>;

    __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][BC * KSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][BC * VSTR];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    // work items as in fa_fwd_16bit_kernel: causal tiles i and n_qtiles-1-i form one item
    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int n_items = CAUSAL ? (n_qtiles + 1) / 2 : n_qtiles;
    const int bh = id / n_items;
    const int item = id % n_items;
    const int n_pass = (CAUSAL && n_qtiles - 1 - item != item) ? 2 : 1;

    const size_t head_off = (size_t)bh * N * D;
    const size_t kv_off = (size_t)(bh / kv_group) * N * D;
    const uint16_t* qh = q + head_off;
    const float sc = scale * kLog2e;
    const __amdgpu_buffer_rsrc_t k_rsrc = make_buffer(k + kv_off, (uint32_t)N * D * 2);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_buffer(v + kv_off, (uint32_t)N * D * 2);
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    const int qt = CAUSAL ? (pass == 0 ? n_qtiles - 1 - item : item) : item;  // the longer tile first
    const int wave_q0 = qt * BR + wave * 32;
    const int limit = CAUSAL ? min(wave_q0 + col, N - 1) : N - 1;  // last key this lane's query sees

    // Q_i^T as the B operand of S^T = K Q^T, resident for the whole loop
    i32x4 qreg[KS];
    {
        const int row = min(wave_q0 + col, N - 1);  // rows past N compute a copy of row N-1, never stored
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qreg[ks] = *reinterpret_cast<const i32x4*>(qh + (size_t)row * D + ks * 16 + half * 8);
    }
    f32x16 oacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f, mb = 0.f;

    const int last_q = min(qt * BR + BR, N) - 1;
    const int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);

    // ---- pieces shared by the prologue and the loop
    float mxp[4];
    auto need_mask = [&](int t) { return (t * BC + BC > N) || (CAUSAL && t * BC + BC - 1 > wave_q0); };
    auto mask_block = [&](int t, f32x16 (&s)[2]) {  // keys past N, and keys after the query when causal
        // compile-time key offsets against one per-lane bound (kept opaque: the compiler otherwise gives the
        // 32 per-element key indices registers of their own)
        int bound = limit - t * BC - 4 * half;
        asm volatile("" : "+v"(bound));
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (kt * 32 + 8 * (r >> 2) + (r & 3) > bound) s[kt][r] = -INFINITY;
    };
    auto max_part = [&](f32x16 (&s)[2], int part) {  // registers 8 part .. 8 part + 7 of the 32
#pragma unroll
        for (int i = 8 * part; i < 8 * part + 8; ++i)
            mxp[i & 3] = i < 4 ? s[0][i] : fmaxf(mxp[i & 3], s[i >> 4][i & 15]);
    };
    // K rows for S^T (A operand), 32 steps (kt, ks); the scores land in ordinary registers
    auto score_step = [&](f32x16 (&s)[2], uint32_t k_rows, i32x4 (&abuf)[KP], int u) {
        constexpr int NU = 2 * KS;
        const int kt = u / KS, ks = u % KS;
        const i32x4 a = abuf[u % KP];
        if (u + KP < NU) {
            const int w = u + KP;
            abuf[u % KP] = lds_load_16B(k_rows + ((w / KS) * 32 * KSTR + (w % KS) * 16) * 2);
        }
        if (ks == 0) MfmaVgprAcc<Tag>::first(s[kt], a, qreg[ks]);
        else MfmaVgprAcc<Tag>::run(s[kt], a, qreg[ks]);
    };
    auto score_prefetch = [&](uint32_t k_rows, i32x4 (&abuf)[KP]) {
#pragma unroll
        for (int u = 0; u < KP; ++u) abuf[u] = lds_load_16B(k_rows + ((u / KS) * 32 * KSTR + (u % KS) * 16) * 2);
    };

    // Staging, global -> registers -> LDS, one 16-byte chunk per thread at a time.  A block's K and V
    // are 64 KiB, half of what the CU's vector memory path moves in the time of the block's MFMAs:
    // issued in one burst the loads make every wave sit in its own issue for over a thousand
    // cycles.  They are spread over the MFMA steps instead, one chunk every CH_EVERY steps, and
    // each chunk is written to the LDS a stage later, when it has long arrived:
    //   stage A of block t: load K(t+2) chunks          | write the V(t+1) chunks loaded in block t-1
    //   stage B of block t: write those K(t+2) chunks   | load V(t+2) chunks
    // (K(t+2) replaces K(t), last read in block t-1; V(t+1) replaces V(t-1), last read in block t-1;
    // both become visible at the barrier that ends block t.)  Blocks past the end read as zero.
    constexpr int NCH = Copy::kPerThread, CH_EVERY = 2 * KS / NCH;
    static_assert(NCH * CH_EVERY == 2 * KS && 4 * DT == 2 * KS, "one chunk every CH_EVERY steps of either stage");
    i32x4 kpre[NCH], vpre[NCH];
    auto load_chunk = [&](__amdgpu_buffer_rsrc_t rsrc, int block_idx, int i) {
        return buffer_load_16B(rsrc, block_idx * BC * D * 2 + (tid + i * NT) * 16);
    };
    auto store_chunk = [&](uint16_t* lds, int stride, int i, const i32x4& x) {
        const int c = tid + i * NT;
        *reinterpret_cast<i32x4*>(lds + (c / (D / 8)) * stride + (c % (D / 8)) * 8) = x;
    };
    Copy::from_global(k_rsrc, 0, tid, kpre);
    Copy::from_global(v_rsrc, 0, tid, vpre);
    Copy::template to_lds<KSTR>(lds_k[0], tid, kpre);
    Copy::template to_lds<VSTR>(lds_v[0], tid, vpre);
    Copy::from_global(k_rsrc, BC * D * 2, tid, kpre);  // K(1)
    Copy::from_global(v_rsrc, BC * D * 2, tid, vpre);  // V(1), written to the LDS during block 0
    // the Q loads complete here and Q moves to the accumulation half
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(qreg[ks]));
    __syncthreads();

    // ---- prologue: S(0) and its reference maximum (O and l are still zero: nothing to rescale)
    f32x16 sa[2], sb[2];
    {
        uint32_t k_rows = lds_address(lds_k[0]) + (col * KSTR + half * 8) * 2;
        asm volatile("" : "+v"(k_rows));
        i32x4 abuf[KP];
        score_prefetch(k_rows, abuf);
#pragma unroll
        for (int u = 0; u < 2 * KS; ++u) {
            score_step(sa, k_rows, abuf, u);
            __builtin_amdgcn_sched_barrier(0);
        }
        Copy::template to_lds<KSTR>(lds_k[1], tid, kpre);
        mfma_result_wait(sa[0], sa[1]);
        if (need_mask(0)) mask_block(0, sa);
#pragma unroll
        for (int part = 0; part < 4; ++part) max_part(sa, part);
        m_run = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3])));
        mb = m_run * sc;
    }
    __syncthreads();

    // ---- one key block: `cur` holds S(t), `nxt` receives S(t+1)
    auto block = [&](int t, f32x16 (&cur)[2], f32x16 (&nxt)[2]) {
        i32x4 pb[4];  // P~(t)^T as B operands, 16 keys each
        float psum = 0.f;
        uint32_t k_rows = lds_address(lds_k[(t + 1) & 1]) + (col * KSTR + half * 8) * 2;
        uint32_t v_tr = lds_address(lds_v[t & 1]) + ((4 * half + tr_row) * VSTR + tr_col) * 2;
        asm volatile("" : "+v"(k_rows), "+v"(v_tr));

        // ---- stage A
        {
            i32x4 abuf[KP];
            score_prefetch(k_rows, abuf);
#pragma unroll
            for (int u = 0; u < 2 * KS; ++u) {
                score_step(nxt, k_rows, abuf, u);
                if (u % CH_EVERY == 0) {
                    store_chunk(lds_v[(t + 1) & 1], VSTR, u / CH_EVERY, vpre[u / CH_EVERY]);
                    kpre[u / CH_EVERY] = load_chunk(k_rsrc, t + 2, u / CH_EVERY);
                }
                if (u == 0) {
                    // Reference maximum for S(t) from the row maxima taken beside the previous block's
                    // products: raised only when they exceed it by more than 2^kLazyLog2 (P~ <= 2^kLazyLog2
                    // otherwise and the factor cancels in O / l).  Every product of the previous block has
                    // been issued, and the MFMAs of this stage write the score registers only, so the rare
                    // rescale of O is in order here.  (Block 0: the prologue has set the reference; no rise.)
                    const float mx = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3])));
                    const bool raise = (mx - m_run) * sc > kLazyLog2;
                    if (__builtin_amdgcn_ballot_w64(raise) != 0) {
                        const float corr = raise ? fast_exp2((m_run - mx) * sc) : 1.0f;
                        m_run = raise ? mx : m_run;
                        l_run *= corr;
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[dt][r] *= corr;
                    }
                    mb = m_run * sc;
                }
#pragma unroll
                for (int c = 0; c < 16; ++c)
                    if (2 + (c * 30) / 16 == u) {  // pair c of the 16: two scores of S(t) become one packed register of P~
                        const int kt = c / 8, j = c % 8;
                        const float p0 = fast_exp2(__builtin_fmaf(cur[kt][2 * j], sc, -mb));
                        const float p1 = fast_exp2(__builtin_fmaf(cur[kt][2 * j + 1], sc, -mb));
                        psum += p0 + p1;
                        pb[2 * kt + (j >> 2)][j & 3] = E::pack2(p0, p1);
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
            l_run += psum;
        }

        // ---- stage B
        {
            constexpr int NU = 4 * DT;  // (16-key slab, d-tile)
            auto v_addr = [&](int u, int hi) -> uint32_t {
                return v_tr + (((u / DT) * 16 + hi * 8) * VSTR + (u % DT) * 32) * 2;
            };
            i32x2 lo[KP], hi[KP];
#pragma unroll
            for (int u = 0; u < KP; ++u) {
                lo[u] = lds_read_tr16(v_addr(u, 0));
                hi[u] = lds_read_tr16(v_addr(u, 1));
            }
            const bool mask_next = need_mask(t + 1);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int sl = u / DT, dt = u % DT;
                const i32x4 a = {lo[u % KP][0], lo[u % KP][1], hi[u % KP][0], hi[u % KP][1]};
                if (u + KP < NU) {
                    lo[u % KP] = lds_read_tr16(v_addr(u + KP, 0));
                    hi[u % KP] = lds_read_tr16(v_addr(u + KP, 1));
                }
                oacc[dt] = E::mma(a, pb[sl], oacc[dt]);
                if (u == 0) mfma_result_wait(nxt[0], nxt[1]);  // written by MFMAs the hazard checker cannot see
                if (u == 1 && mask_next) mask_block(t + 1, nxt);
                if (u >= 2 && u < 6) max_part(nxt, u - 2);
                if (u % CH_EVERY == 0) {
                    store_chunk(lds_k[t & 1], KSTR, u / CH_EVERY, kpre[u / CH_EVERY]);
                    vpre[u / CH_EVERY] = load_chunk(v_rsrc, t + 2, u / CH_EVERY);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        __syncthreads();
    };

    for (int t = 0; t < n_blocks; t += 2) {
        block(t, sa, sb);
        if (t + 1 < n_blocks) block(t + 1, sb, sa);
    }

    // ---- epilogue: O / l, L = m + log l, through a 4 KiB LDS patch per wave (the last barrier of
    // the loop has passed, so the K buffers are free)
    {
        char* patch = reinterpret_cast<char*>(&lds_k[0][0]) + wave * 4096;
        static_assert(sizeof(lds_k) >= 4 * 4096, "patches must fit");
        const int qi = wave_q0 + col;
        const float l = sum_both_halves(l_run);
        store_rows_via_lds<Tag, DT>(oacc, 1.0f / l, patch, make_buffer(o + head_off, (uint32_t)N * D * 2), wave_q0, lane);
        if (qi < N && half == 0) lse[(size_t)bh * N + qi] = (m_run * sc + log2f(l)) * kLn2;
    }
    if (pass + 1 < n_pass) __syncthreads();  // the next pass's first tile overwrites the patches
    }  // passes of a causal pair
}

// ---------------------------------------------------------------------------------------
// Eight-wave ping-pong variant (head dimension 128).
//
// An eight-wave workgroup puts two waves on every SIMD (waves w and w + 4).  If all of them run
// a block's steps in the same order they stay in lock-step: both waves of a SIMD issue MFMAs
// together and then both do softmax together, so the matrix pipe idles during every softmax --
// the problem the paper's ping-pong scheduling (section 3.1) solves with named barriers between
// two warpgroups.  Here the waves form two groups, one wave of each per SIMD, and every
// iteration has two half-steps separated by workgroup barriers:
//
//     iteration t          half-step 1                   half-step 2
//        group A     MFMA stream(t)                 softmax(t), operand prefetch
//        group B     softmax(t-1), prefetch         MFMA stream(t)
//
//     stream(t) = O^T += V(t-1)^T P~(t-1)^T  followed by  S(t)^T = K(t) Q^T
//
// so that one wave of each SIMD always has MFMA work while the other has VALU work.  Group A
// carries P~ from one iteration to the next, group B carries S.  A stream is one sequence of
// (LDS operand read, MFMA) units whose reads run P units ahead of their use through a register
// ring; the first P reads are issued before the barrier that precedes the stream, so they
// complete while the wave waits there.
//
// Staging: K and V blocks go from global memory straight into a ring of NS LDS stages
// (buffer loads with an LDS destination: no staging registers, no LDS store instructions), issued
// two to three iterations before their first use.  Such a load writes 64 lanes x 16 bytes
// contiguously, so the tiles are stored unpadded (256 bytes per row) and bank conflicts are
// avoided by an XOR swizzle of the 16-byte chunk index instead, applied through the *global*
// address each lane fetches:  K: chunk ^ (row % 16)  (16 lanes read 16 rows at one chunk),
// V: chunk ^ 4 (row % 4)  (a transposing read covers 4 rows x 4 chunks).
template <typename Tag, int BC, int P, bool CAUSAL>
__global__ void __launch_bounds__(512, 2)
fa_fwd_pingpong_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k,
                       const uint16_t* __restrict__ v, uint16_t* __restrict__ o, float* __restrict__ lse,
                       int N, int n_qtiles, int total_wg, int kv_group, float scale) {
    [[maybe_unused]] ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int D = 128;
    constexpr int BR = 256;
    constexpr int NS = 4;              // LDS stages per tensor
    constexpr int ROWB = D * 2;        // bytes per tile row
    constexpr int TILE = BC * ROWB;    // bytes per stage
    constexpr int KT = BC / 32;
    constexpr int KS = D / 16;
    constexpr int DT = D / 32;
    constexpr int SL = BC / 16;
    constexpr int N1 = SL * DT;  // MFMA units of the second GEMM
    constexpr int N0 = KS * KT;  // MFMA units of the first GEMM
    static_assert(BC == 64, "the staging pattern below covers 64-row tiles with two loads per wave");
    using E = Elem<Tag>;

    __shared__ __attribute__((aligned(1024))) char lds_k[NS * TILE];
    __shared__ __attribute__((aligned(1024))) char lds_v[NS * TILE];
    __shared__ __attribute__((aligned(1024))) char lds_o[8 * 4096];  // output transposition, 4 KiB per wave

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;
    // the two waves of a SIMD take adjacent 32-row slabs of the query tile
    const int group = wave >> 2;
    const int slab = (wave & 3) * 2 + group;

    // Work items.  Non-causal: one query tile.  Causal: query tiles i and n_qtiles-1-i of a head,
    // one after the other -- every item then covers the same number of key blocks, so the grid
    // has no long and short workgroups and no tail of stragglers (with an odd tile count the
    // middle tile is an item of its own).
    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int n_items = CAUSAL ? (n_qtiles + 1) / 2 : n_qtiles;
    const int bh = id / n_items;
    const int item = id % n_items;
    const int n_pass = (CAUSAL && n_qtiles - 1 - item != item) ? 2 : 1;

    const size_t head_off = (size_t)bh * N * D;
    const uint16_t* qh = q + head_off;
    int wave_q0 = 0;  // first query row of this wave in the current pass
    const float sc = scale * kLog2e;
    float sc_v = sc;  // a vector-register copy: an FMA with a scalar-register operand issues at a lower rate
    asm volatile("" : "+v"(sc_v));

    i32x4 qreg[KS];
    f32x16 oacc[DT];
    float m_run = 0.f, l_run = 0.f;  // reference (log2 units of the scaled scores) and row sum of P~

    // ---- staging: wave w loads rows 4w .. 4w+3 and 32+4w .. 32+4w+3 of a tile (1 KiB each)
    const size_t kv_off = (size_t)(bh / kv_group) * N * D;  // grouped-query: kv_group query heads per K/V head
    const BufferWords k_rsrc = make_buffer_words(k + kv_off, (uint32_t)N * D * 2);
    const BufferWords v_rsrc = make_buffer_words(v + kv_off, (uint32_t)N * D * 2);
    const int st_row = 4 * wave + (lane >> 4), st_pos = lane & 15;
    const int k_src = st_row * ROWB + ((st_pos ^ (st_row & 15)) << 4);        // byte offset within a tile
    const int v_src = st_row * ROWB + ((st_pos ^ ((st_row & 3) << 2)) << 4);
    const uint32_t lds_k0 = (uint32_t)(uintptr_t)lds_k + wave * 1024, lds_v0 = (uint32_t)(uintptr_t)lds_v + wave * 1024;
    // Block u of K and block u2 of V.  Blocks past the end lie outside the buffer resources and
    // read as zeros, so every iteration issues the same four loads and the vmcnt waits below can
    // count on that.
    auto stage_k = [&](int u) __attribute__((always_inline)) {
        const uint32_t kd = lds_k0 + (u & (NS - 1)) * TILE;
        global_to_lds_16B(k_rsrc, kd, k_src + u * TILE);
        global_to_lds_16B(k_rsrc, kd + 8 * 1024, k_src + u * TILE + 32 * ROWB);
    };
    auto stage_v = [&](int u) __attribute__((always_inline)) {
        const uint32_t vd = lds_v0 + (u & (NS - 1)) * TILE;
        global_to_lds_16B(v_rsrc, vd, v_src + u * TILE);
        global_to_lds_16B(v_rsrc, vd + 8 * 1024, v_src + u * TILE + 32 * ROWB);
    };
    auto stage = [&](int u, int u2) __attribute__((always_inline)) {
        stage_k(u);
        stage_v(u2);
    };

    // ---- per-lane operand offsets within a stage (bytes)
    const int tr_row = (lane & 15) >> 2, quad = lane & 3, blk = (lane >> 4) & 1;
    int kofs[KS], vofs[DT];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) kofs[ks] = col * ROWB + (((2 * ks + half) ^ (col & 15)) << 4);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
        vofs[dt] = (4 * half + tr_row) * ROWB + (((4 * dt + 2 * blk + (quad >> 1)) ^ (tr_row << 2)) << 4) + 8 * (quad & 1);

    f32x16 sacc[KT];
    i32x4 pb[SL];
    i32x4 ring[P];

    // Unit u of stream(t): the second GEMM's units (if DO1) then the first GEMM's (if DO0).
    auto read_unit = [&](auto do1, int t, int u) __attribute__((always_inline)) {
        constexpr int n1 = decltype(do1)::value ? N1 : 0;
        if (u < n1) {
#if FA_ABLATE_PP == 2
            asm volatile("" : "+v"(ring[u % P]));
#else
            const int sl = u / DT, dt = u % DT;
            const char* p0 = lds_v + ((t - 1) & (NS - 1)) * TILE + vofs[dt] + sl * 16 * ROWB;
            i32x2 lo = lds_read_tr16(p0);
            i32x2 hi = lds_read_tr16(p0 + 8 * ROWB);
            ring[u % P] = i32x4{lo[0], lo[1], hi[0], hi[1]};
#endif
        } else {
#if FA_ABLATE_PP == 3
            asm volatile("" : "+v"(ring[u % P]));
#else
            const int ks = (u - n1) / KT, kt = (u - n1) % KT;
            ring[u % P] = *reinterpret_cast<const i32x4*>(lds_k + (t & (NS - 1)) * TILE + kofs[ks] + kt * 32 * ROWB);
#endif
        }
    };
    auto prefill = [&](auto do1, auto do0, int t) __attribute__((always_inline)) {
        constexpr int NU = (decltype(do1)::value ? N1 : 0) + (decltype(do0)::value ? N0 : 0);
#pragma unroll
        for (int u = 0; u < (P < NU ? P : NU); ++u) read_unit(do1, t, u);
    };
    auto run_stream = [&](auto do1, auto do0, int t) __attribute__((always_inline)) {
        constexpr int n1 = decltype(do1)::value ? N1 : 0;
        constexpr int NU = n1 + (decltype(do0)::value ? N0 : 0);
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const i32x4 a = ring[u % P];
            if (u + P < NU) read_unit(do1, t, u + P);
            if (u < n1) {
                const int sl = u / DT, dt = u % DT;
                oacc[dt] = E::mma(a, pb[sl], oacc[dt]);
            } else {
                const int ks = (u - n1) / KT, kt = (u - n1) % KT;
                sacc[kt] = E::mma(a, qreg[ks], ks == 0 ? zero : sacc[kt]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // mask block t (keys past N; keys after the query when causal), then the online softmax of
    // Algorithm 1 (m, P~, l); P~ leaves packed as the B operand of the second GEMM
    auto softmax = [&](int t) __attribute__((always_inline)) {
        const int key0 = t * BC;
        if ((key0 + BC > N) || (CAUSAL && key0 + BC - 1 > wave_q0)) {
            const int qi = wave_q0 + col;
            const int limit = CAUSAL ? min(qi, N - 1) : N - 1;  // last visible key
            // compile-time key offsets against one opaque per-lane bound: a compare and a select per score
            int bound = limit - key0 - 4 * half;
            asm volatile("" : "+v"(bound));
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kt * 32 + 8 * (r >> 2) + (r & 3) > bound) sacc[kt][r] = -INFINITY;
        }
        // Every step below is a batch of independent instructions: a wave gets few issue slots
        // while its SIMD sibling streams MFMAs, and dependent chains (fma -> exp, sum) would turn
        // each slot missed into a stall.
        //
        // No row maximum is taken per block.  Scores are referred to a per-row reference m (log2
        // units) that is the true row maximum of block 0 and afterwards moves only when a block's
        // P~ grow large: x = s c - m stays in the score registers, P~ = exp2(x) goes to the operand
        // registers, and the block's row sum -- needed anyway -- is the overflow detector.  While it
        // stays below kRaiseAbove every P~ of the block is below it too (also the 16-bit P~ of the
        // fp16 path); otherwise the reference is moved to this block's true maximum, O and l are
        // rescaled and the block's P~ recomputed from x.  The reference cancels in O / l and L is
        // m + log2 l either way, so the result is that of Algorithm 1 with any reference.
#if FA_ABLATE_PP != 4
#pragma unroll
        for (int kt = 0; kt < KT; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[kt][r] = __builtin_fmaf(sacc[kt][r], sc_v, -m_run);
#endif
        __builtin_amdgcn_sched_barrier(0);
        float blk = 0.f;
        auto probabilities = [&]() __attribute__((always_inline)) {
            float ps[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                float e[16];
#pragma unroll
#if FA_ABLATE_PP == 1 || FA_ABLATE_PP == 4
                for (int r = 0; r < 16; ++r) e[r] = sacc[kt][r];
#else
                for (int r = 0; r < 16; ++r) e[r] = fast_exp2(sacc[kt][r]);
#endif
#if FA_ABLATE_PP != 4
#pragma unroll
                for (int r = 0; r < 16; ++r) ps[r & 3] += e[r];
#endif
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    i32x4 w;
#pragma unroll
                    for (int i = 0; i < 4; ++i) w[i] = E::pack2(e[8 * s2 + 2 * i], e[8 * s2 + 2 * i + 1]);
                    pb[2 * kt + s2] = w;
                }
            }
            blk = (ps[0] + ps[1]) + (ps[2] + ps[3]);
        };
        probabilities();
        const bool first = t == 0;
        const bool raise = first || max_both_halves(blk) > kRaiseAbove;
        if (first || __builtin_amdgcn_ballot_w64(raise) != 0) {
            float mxp[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) mxp[c] = sacc[0][c];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) mxp[r & 3] = fmaxf(mxp[r & 3], sacc[kt][r]);
            const float mx = max_both_halves(fmaxf(fmaxf(mxp[0], mxp[1]), fmaxf(mxp[2], mxp[3])));
            const float delta = raise ? mx : 0.f;
            const float corr = fast_exp2(-delta);
            m_run += delta;
            l_run *= corr;
            if (!first) {
#pragma unroll
                for (int dt = 0; dt < DT; ++dt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[dt][r] *= corr;
            }
#pragma unroll
            for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                for (int r = 0; r < 16; ++r) sacc[kt][r] -= delta;
            probabilities();
        }
        l_run += blk;
        // P~ must exist in registers here: the compiler is otherwise free to sink the exponentials
        // past the next barrier, next to the MFMAs that consume them
#pragma unroll
        for (int i = 0; i < SL; ++i) asm volatile("" : "+v"(pb[i]));
    };

    // Workgroup barrier that leaves the staging loads in flight.  LDS reads issued before it (the
    // operand prefetch) may still be outstanding; their results are only used after it anyway.
    auto barrier = [&]() __attribute__((always_inline)) {
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        __builtin_amdgcn_sched_barrier(0);
    };
    // Iteration t issues K(t+3) and V(t+2) (four loads per wave); before the barrier that ends
    // half-step 1 of iteration t a wave makes sure its loads of iteration t-2 have landed: K(t+1)
    // and V(t), first read by the prefetch at the end of this iteration.
    auto mid_barrier = [&]() __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        barrier();
    };

    const std::true_type yes{};
    const std::false_type no{};

#pragma nounroll
    for (int pass = 0; pass < n_pass; ++pass) {
    const int qt = CAUSAL ? (pass == 0 ? n_qtiles - 1 - item : item) : item;  // the longer tile first
    wave_q0 = qt * BR + slab * 32;
    {
        int row = min(wave_q0 + col, N - 1);  // rows past N compute a copy of row N-1, never stored
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            qreg[ks] = *reinterpret_cast<const i32x4*>(qh + (size_t)row * D + ks * 16 + half * 8);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
    m_run = 0.f;  // set from block 0's row maximum by its softmax
    l_run = 0.f;
    const int last_q = min(qt * BR + BR, N) - 1;
    const int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);
    // blocks 0 .. nb_w-1 concern this wave (all of them unless causal)
    const int nb_w = CAUSAL ? min(n_blocks, (wave_q0 + 31) / BC + 1) : n_blocks;
    // every wave's staging loads of the previous pass have landed (each waited for its own
    // before its epilogue) and every LDS read of that pass is done
    if (pass > 0) barrier();

    // ---- prologue: K(0), K(1), K(2), V(0), V(1) staged and visible before the first iteration
    stage(0, 0);
    stage(1, 1);
    stage_k(2);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qreg[ks]));  // Q loads complete before the loop
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    barrier();

    if (group == 0) {
        prefill(no, yes, 0);
        // stream(t) was prefetched at the end of the previous iteration
        auto iteration = [&](int t, auto do1, auto do0, auto next1, auto next0) __attribute__((always_inline)) {
            stage(t + 3, t + 2);
            run_stream(do1, do0, t);
            mid_barrier();
            if constexpr (decltype(do0)::value) softmax(t);
            prefill(next1, next0, t + 1);
            barrier();
        };
        // stream shapes over t: (no,yes) at 0; (yes,yes) for 1..nb_w-1; (yes,no) at nb_w; nothing after
        if (nb_w > 1) iteration(0, no, yes, yes, yes);
        else iteration(0, no, yes, yes, no);
        for (int t = 1; t + 1 < nb_w; ++t) iteration(t, yes, yes, yes, yes);
        if (nb_w > 1) iteration(nb_w - 1, yes, yes, yes, no);
        iteration(nb_w, yes, no, no, no);
        for (int t = nb_w + 1; t <= n_blocks; ++t) iteration(t, no, no, no, no);
    } else {
        auto iteration = [&](int t, auto do1, auto do0) __attribute__((always_inline)) {
            stage(t + 3, t + 2);
            prefill(do1, do0, t);
            if constexpr (decltype(do1)::value) softmax(t - 1);
            mid_barrier();
            run_stream(do1, do0, t);
            barrier();
        };
        iteration(0, no, yes);
        for (int t = 1; t < nb_w; ++t) iteration(t, yes, yes);
        iteration(nb_w, yes, no);
        for (int t = nb_w + 1; t <= n_blocks; ++t) iteration(t, no, no);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // staging loads past the last block: nothing may land after the end

    // ---- epilogue: O / l, L = m + log l
    {
        const int qi = wave_q0 + col;
        const float l = sum_both_halves(l_run);
        store_rows_via_lds<Tag, DT>(oacc, 1.0f / l, lds_o + wave * 4096, make_buffer(o + head_off, (uint32_t)N * D * 2),
                                    wave_q0, lane);
        if (qi < N && half == 0) lse[(size_t)bh * N + qi] = (m_run + log2f(l)) * kLn2;
    }
    }  // passes of a causal pair
}

// ---------------------------------------------------------------------------------------
// fp32 path (d = 64): plain fp32 FMA arithmetic with the same structure -- a query tile per
// workgroup, K/V blocks staged in LDS, online softmax with exp2 and the scale folded in.
// One thread owns one query row, so no cross-lane reductions are needed.
template <int D, int BC, bool CAUSAL>
__global__ void __launch_bounds__(64) fa_fwd_f32_kernel(const float* __restrict__ q, const float* __restrict__ k,
                                                        const float* __restrict__ v, float* __restrict__ o,
                                                        float* __restrict__ lse, int N, int n_qtiles, int kv_group,
                                                        float scale) {
    constexpr int BR = 64;
    __shared__ float lds_k[BC * D];
    __shared__ float lds_v[BC * D];
    const int tid = threadIdx.x;
    const int bh = blockIdx.x / n_qtiles, qt = blockIdx.x % n_qtiles;
    const size_t head_off = (size_t)bh * N * D;
    const size_t kv_off = (size_t)(bh / kv_group) * N * D;
    const int qi = qt * BR + tid;
    const float sc = scale * kLog2e;

    float qr[D], acc[D];
#pragma unroll
    for (int c = 0; c < D; ++c) {
        qr[c] = qi < N ? q[head_off + (size_t)qi * D + c] : 0.f;
        acc[c] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;
    int last_q = min(qt * BR + BR, N) - 1;
    int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);
    for (int t = 0; t < n_blocks; ++t) {
        int key0 = t * BC;
        __syncthreads();
        for (int e = tid; e < BC * D; e += 64) {
            int key = key0 + e / D;
            lds_k[e] = key < N ? k[kv_off + (size_t)key0 * D + e] : 0.f;
            lds_v[e] = key < N ? v[kv_off + (size_t)key0 * D + e] : 0.f;
        }
        __syncthreads();
        float s[BC];
        float mx = -INFINITY;
        int limit = CAUSAL ? min(qi, N - 1) : N - 1;
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            float a = 0.f;
#pragma unroll
            for (int c = 0; c < D; ++c) a = __builtin_fmaf(qr[c], lds_k[j * D + c], a);
            s[j] = (key0 + j > limit) ? -INFINITY : a;
            mx = fmaxf(mx, s[j]);
        }
        float m_new = fmaxf(m_run, mx);
        if (m_new == -INFINITY) continue;  // row past N in a causal tail: nothing visible yet
        float corr = fast_exp2((m_run - m_new) * sc);
        m_run = m_new;
        float mb = m_new * sc;
        l_run *= corr;
#pragma unroll
        for (int c = 0; c < D; ++c) acc[c] *= corr;
#pragma unroll
        for (int j = 0; j < BC; ++j) {
            float p = fast_exp2(__builtin_fmaf(s[j], sc, -mb));
            l_run += p;
#pragma unroll
            for (int c = 0; c < D; ++c) acc[c] = __builtin_fmaf(p, lds_v[j * D + c], acc[c]);
        }
    }
    if (qi < N) {
        float inv = 1.0f / l_run;
#pragma unroll
        for (int c = 0; c < D; ++c) o[head_off + (size_t)qi * D + c] = acc[c] * inv;
        lse[(size_t)bh * N + qi] = (m_run * sc + log2f(l_run)) * kLn2;
    }
}

// ---------------------------------------------------------------------------------------
template <typename Tag, int D, int BC, int NW, int RQ, int PD>
static int launch_16bit(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N,
                        float scale, int causal, hipStream_t stream) {
    constexpr int BR = NW * 32 * RQ;
    int n_qtiles = (N + BR - 1) / BR;
    long total = (long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);  // causal: tiles are paired up
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(NW * 64);
    auto qp = static_cast<const uint16_t*>(q);
    auto kp = static_cast<const uint16_t*>(k);
    auto vp = static_cast<const uint16_t*>(v);
    auto op = static_cast<uint16_t*>(o);
    if (causal)
        hipLaunchKernelGGL((fa_fwd_16bit_kernel<Tag, D, BC, NW, RQ, PD, true>), grid, block, 0, stream, qp, kp, vp,
                           op, lse, N, n_qtiles, (int)total, H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_fwd_16bit_kernel<Tag, D, BC, NW, RQ, PD, false>), grid, block, 0, stream, qp, kp, vp,
                           op, lse, N, n_qtiles, (int)total, H / H_kv, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

template <typename Tag>
static int launch_pingpong(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N,
                           float scale, int causal, hipStream_t stream) {
    constexpr int BR = 256, BC = 64, P = 4;
    int n_qtiles = (N + BR - 1) / BR;
    long total = (long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);  // causal: tiles are paired up
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(512);
    auto qp = static_cast<const uint16_t*>(q);
    auto kp = static_cast<const uint16_t*>(k);
    auto vp = static_cast<const uint16_t*>(v);
    auto op = static_cast<uint16_t*>(o);
    if (causal)
        hipLaunchKernelGGL((fa_fwd_pingpong_kernel<Tag, BC, P, true>), grid, block, 0, stream, qp, kp, vp, op, lse, N,
                           n_qtiles, (int)total, H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_fwd_pingpong_kernel<Tag, BC, P, false>), grid, block, 0, stream, qp, kp, vp, op, lse, N,
                           n_qtiles, (int)total, H / H_kv, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

template <typename Tag>
static int launch_d256(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N,
                       float scale, int causal, hipStream_t stream) {
    constexpr int BR = 128;
    int n_qtiles = (N + BR - 1) / BR;
    long total = (long)B * H * (causal ? (n_qtiles + 1) / 2 : n_qtiles);  // causal: tiles are paired up
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(256);
    auto qp = static_cast<const uint16_t*>(q);
    auto kp = static_cast<const uint16_t*>(k);
    auto vp = static_cast<const uint16_t*>(v);
    auto op = static_cast<uint16_t*>(o);
    if (causal)
        hipLaunchKernelGGL((fa_fwd_d256_kernel<Tag, true>), grid, block, 0, stream, qp, kp, vp, op, lse, N, n_qtiles,
                           (int)total, H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_fwd_d256_kernel<Tag, false>), grid, block, 0, stream, qp, kp, vp, op, lse, N, n_qtiles,
                           (int)total, H / H_kv, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

// Kernel choice (measured on MI355X at the 16k-token benchmark shapes):
//   d = 128: the eight-wave ping-pong kernel for long sequences (causal tiles are paired into
//     items of equal length there, so its coarser tiles cost no balance); shorter problems keep
//     128-row workgroups of four waves, which fill the chip better and waste less of a tile on
//     the diagonal.  The two cross between 640 and 768 keys without a mask and near 1400 with one
//     (measured at 16k and 64k tokens per launch).
//   d = 64: eight waves share each K/V block (256 query rows per workgroup, two waves per SIMD),
//     four waves for short problems (crossover near 700 keys without a mask, 1300 with one).
//   d = 256: the 128-register output accumulator allows only one wave per SIMD; fa_fwd_d256_kernel
//     pipelines the softmax of one block under the score MFMAs of the next inside that wave.
enum class Fwd16 { kTile4, kTile8, kPingPong, kD256, kNone };
static Fwd16 choose_16bit(int d, int N, int causal) {
    switch (d) {
        case 64: return N <= (causal ? 1280 : 640) ? Fwd16::kTile4 : Fwd16::kTile8;
        case 128: return N <= (causal ? 1408 : 640) ? Fwd16::kTile4 : Fwd16::kPingPong;
        case 256: return Fwd16::kD256;
        default: return Fwd16::kNone;
    }
}

template <typename Tag>
static int dispatch_16bit(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N,
                          int d, float scale, int causal, int schedule, hipStream_t stream) {
    if (schedule != FA_SCHED_AUTO) {
        // forced kernel choice for the scheduling ablation (section 4.2's table, re-done on this chip)
        if (d != 128) return FA_ERR_UNSUPPORTED;
        switch (schedule) {
            case FA_SCHED_LOCKSTEP_4W:
                return launch_16bit<Tag, 128, 64, 4, 1, 0>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
            case FA_SCHED_LOCKSTEP_8W:
                return launch_16bit<Tag, 128, 128, 8, 1, 0>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
            case FA_SCHED_PINGPONG: return launch_pingpong<Tag>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
            default: return FA_ERR_SHAPE;
        }
    }
    switch (choose_16bit(d, N, causal)) {
        case Fwd16::kTile4:
            if (d == 64) return launch_16bit<Tag, 64, 64, 4, 1, 0>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
            return launch_16bit<Tag, 128, 64, 4, 1, 0>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
        case Fwd16::kTile8: return launch_16bit<Tag, 64, 64, 8, 1, 0>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
        case Fwd16::kPingPong: return launch_pingpong<Tag>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
        case Fwd16::kD256: return launch_d256<Tag>(q, k, v, o, lse, B, H, H_kv, N, scale, causal, stream);
        default: return FA_ERR_UNSUPPORTED;
    }
}

// The name a profiler shows for the kernel dispatch_16bit picks (FA_SCHED_AUTO).
const char* fwd_16bit_kernel_name(bool f16, int N, int d, int causal) {
    static const char* const names[2][2][5] = {
        {{"fa_fwd_16bit_kernel<bf16_tag, 64, 64, 4, 1, 0, false>", "fa_fwd_16bit_kernel<bf16_tag, 128, 64, 4, 1, 0, false>",
          "fa_fwd_16bit_kernel<bf16_tag, 64, 64, 8, 1, 0, false>", "fa_fwd_pingpong_kernel<bf16_tag, 64, 4, false>",
          "fa_fwd_d256_kernel<bf16_tag, false>"},
         {"fa_fwd_16bit_kernel<bf16_tag, 64, 64, 4, 1, 0, true>", "fa_fwd_16bit_kernel<bf16_tag, 128, 64, 4, 1, 0, true>",
          "fa_fwd_16bit_kernel<bf16_tag, 64, 64, 8, 1, 0, true>", "fa_fwd_pingpong_kernel<bf16_tag, 64, 4, true>",
          "fa_fwd_d256_kernel<bf16_tag, true>"}},
        {{"fa_fwd_16bit_kernel<f16_tag, 64, 64, 4, 1, 0, false>", "fa_fwd_16bit_kernel<f16_tag, 128, 64, 4, 1, 0, false>",
          "fa_fwd_16bit_kernel<f16_tag, 64, 64, 8, 1, 0, false>", "fa_fwd_pingpong_kernel<f16_tag, 64, 4, false>",
          "fa_fwd_d256_kernel<f16_tag, false>"},
         {"fa_fwd_16bit_kernel<f16_tag, 64, 64, 4, 1, 0, true>", "fa_fwd_16bit_kernel<f16_tag, 128, 64, 4, 1, 0, true>",
          "fa_fwd_16bit_kernel<f16_tag, 64, 64, 8, 1, 0, true>", "fa_fwd_pingpong_kernel<f16_tag, 64, 4, true>",
          "fa_fwd_d256_kernel<f16_tag, true>"}}};
    int idx;
    switch (choose_16bit(d, N, causal)) {
        case Fwd16::kTile4: idx = d == 64 ? 0 : 1; break;
        case Fwd16::kTile8: idx = 2; break;
        case Fwd16::kPingPong: idx = 3; break;
        case Fwd16::kD256: idx = 4; break;
        default: return nullptr;
    }
    return names[f16 ? 1 : 0][causal ? 1 : 0][idx];
}

int launch_fwd_bf16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                    float scale, int causal, int schedule, hipStream_t stream) {
    return dispatch_16bit<bf16_tag>(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, schedule, stream);
}

int launch_fwd_f16(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                   float scale, int causal, int schedule, hipStream_t stream) {
    return dispatch_16bit<f16_tag>(q, k, v, o, lse, B, H, H_kv, N, d, scale, causal, schedule, stream);
}

int launch_fwd_f32(const void* q, const void* k, const void* v, void* o, float* lse, int B, int H, int H_kv, int N, int d,
                   float scale, int causal, hipStream_t stream) {
    if (d != 64) return FA_ERR_UNSUPPORTED;
    constexpr int BR = 64;
    int n_qtiles = (N + BR - 1) / BR;
    long total = (long)B * H * n_qtiles;
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    dim3 grid((unsigned)total), block(64);
    auto qp = static_cast<const float*>(q);
    auto kp = static_cast<const float*>(k);
    auto vp = static_cast<const float*>(v);
    auto op = static_cast<float*>(o);
    if (causal)
        hipLaunchKernelGGL((fa_fwd_f32_kernel<64, 32, true>), grid, block, 0, stream, qp, kp, vp, op, lse, N, n_qtiles,
                           H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_fwd_f32_kernel<64, 32, false>), grid, block, 0, stream, qp, kp, vp, op, lse, N,
                           n_qtiles, H / H_kv, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

}  // namespace fa

FA_CLOCK_SPAN_READER(fa_debug_clock_span_fwd)
