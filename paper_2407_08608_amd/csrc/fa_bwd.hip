// Backward attention for gfx950, head dimensions 64, 128 and 256, bf16 / fp16 (paper section 2.1 chain rule,
// Algorithm 3's recomputation of P from L and its D = rowsum(dO o O)).
//
//   preprocess : D = rowsum(dO o O) per query row (HBM-bound)
//   dK/dV pass : one workgroup per block of 128 keys (wave w owns keys 32w..32w+31 and keeps
//                dK_j, dV_j on chip); loop over tiles of 64 queries:
//                S = Q_i K_j^T, dP = dO_i V_j^T, P = exp(S - L), dS = P o (dP - D),
//                dV_j += P^T dO_i, dK_j += dS^T Q_i
//   dQ pass    : one workgroup per tile of queries (dQ_i on chip), loop over key blocks:
//                S^T = K_j Q_i^T, dP^T = V_j dO_i^T, P, dS as above, dQ_i^T += K_j^T dS^T
//
// Algorithm 3 produces dQ inside the dK/dV loop and adds it to HBM with atomics.  Measured on
// MI355X that accumulation (17 GB of fp32 atomic traffic at seqlen 16k) cost about 30 % of the
// pass, so dQ gets its own pass instead: two of the five GEMMs are recomputed, nothing is
// accumulated in HBM, no fp32 dQ buffer or cast pass exists, and the result is deterministic.
//
// Register layouts.  dK/dV pass: S and dP have queries as MFMA rows and keys as columns, so a
// lane owns one key and 16 queries; packed to 16 bits those registers are directly the A
// operand (keys x queries) of the dV and dK products, whose B operands (dO, Q as queries x d)
// come from transposing LDS reads.  dQ pass: the forward kernel's layout -- S^T and dP^T have
// one query per lane column, dS^T packs straight into the B operand of dQ^T += K^T dS^T, and
// K^T is the transposing read of the same LDS tile that fed S^T.
#include <type_traits>

#include "fa_device.h"
#include "fa_launch.h"

namespace fa {


// LDS row stride (elements) of tiles that are read both by rows and transposed: an odd multiple
// of 16 bytes keeps the row reads conflict-free, and the offset from a multiple of 256 bytes
// decides how much the four rows of a transposing read overlap in the banks.
constexpr int bwd_row_stride(int d) { return d >= 128 ? d + 24 : d + 40; }

// ---------------------------------------------------------------------------------------
template <typename Tag, int D>
__global__ void __launch_bounds__(256)
fa_bwd_preprocess_kernel(const uint16_t* __restrict__ o, const uint16_t* __restrict__ dout,
                         float* __restrict__ dvec, long rows) {
    constexpr int LPR = D / 8;  // lanes per row, 8 elements each
    using E = Elem<Tag>;
    const int lane16 = threadIdx.x & (LPR - 1);
    long row = (long)blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
    float acc = 0.f;
    if (row < rows) {
        i32x4 a = *reinterpret_cast<const i32x4*>(o + row * D + lane16 * 8);
        i32x4 b = *reinterpret_cast<const i32x4*>(dout + row * D + lane16 * 8);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            uint32_t ua = (uint32_t)a[t], ub = (uint32_t)b[t];
            acc = __builtin_fmaf(E::to_float((uint16_t)(ua & 0xFFFF)), E::to_float((uint16_t)(ub & 0xFFFF)), acc);
            acc = __builtin_fmaf(E::to_float((uint16_t)(ua >> 16)), E::to_float((uint16_t)(ub >> 16)), acc);
        }
    }
#pragma unroll
    for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (row < rows && lane16 == 0) dvec[row] = acc;
}

// ---------------------------------------------------------------------------------------
template <typename Tag, int D, bool CAUSAL>
__global__ void __launch_bounds__(256, D >= 128 ? 1 : 2)
fa_bwd_dkdv_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
              const uint16_t* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ dvec,
              uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int N,
              int n_kblocks, int total_wg, int kv_group, float scale) {
    [[maybe_unused]] ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int BK = 128;        // keys per workgroup
    constexpr int BQ = 64;         // queries per loop iteration
    constexpr int NT = 256;
    // Row stride of the Q and dO tiles: they are read both as rows (128-bit) and transposed.
    // Measured LDS rates per CU at D = 128: 304 B gives 211 / 123 B/clk (rows / transposed), 272 B
    // gives 208 / 63, 320 B gives 63 / 208.  (An unpadded XOR-swizzled layout that frees both
    // reads of bank conflicts altogether was measured too: same speed, the kernel is bound by
    // the instruction issue of its one wave per SIMD, not by the LDS.)
    constexpr int RSTR = bwd_row_stride(D);
    constexpr int TILE_B = BQ * RSTR * 2;  // bytes per tile
    constexpr int KS = D / 16;
    // MFMA steps by which LDS operand reads lead their use (registers permitting)
    constexpr int KP = D == 128 ? 4 : 2;
    // The step loops below must be unrolled (register arrays are indexed by the step).  At d = 256
    // with the causal mask the unrolled body passes the size at which "#pragma unroll" gives up
    // silently; this file is compiled with that threshold raised (see build.py).
    // S and dP contract over the whole head dimension; dK and dV are produced for a slice of DO
    // columns per workgroup (the whole of it up to d = 128; at d = 256 two workgroups, blockIdx.y,
    // take half each and both recompute S and dP -- the accumulators of all 256 columns, 256
    // registers per lane on top of the K and V operands, do not fit the register file)
    constexpr int DO = D > 128 ? 128 : D;
    constexpr int DT = DO / 32;
    constexpr int CPR = D / 8;     // 16-byte chunks per row
    constexpr int QCH = BQ * CPR / NT;  // chunks per thread for a Q / dO tile
    // With one wave per SIMD (more than 256 registers per lane) MFMA results land in the
    // accumulation half of the register file unless told otherwise; the score tiles S and dP,
    // which the exponentials read, are then produced by MfmaVgprAcc into ordinary registers.
    constexpr bool VACC = D >= 128;
    using E = Elem<Tag>;
    const int col0 = blockIdx.y * DO;  // first column of this workgroup's slice

    // tiles 0, 1: Q_i double-buffered; tiles 2, 3: dO_i (a fixed distance from the Q tile of the
    // same parity, so one address register serves both)
    __shared__ __attribute__((aligned(16))) uint16_t lds_t[4][BQ * RSTR];
    constexpr int DO_DIST = 2 * TILE_B;
    __shared__ __attribute__((aligned(16))) float lds_l[2][BQ];
    __shared__ __attribute__((aligned(16))) float lds_d[2][BQ];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int bh = id / n_kblocks;
    const int kb = id % n_kblocks;  // causal: key block 0 has the longest loop and comes first
    const int key0 = kb * BK;

    // bh counts key/value heads; the kv_group query heads that share this one are bh * kv_group + g
    const size_t head_off = (size_t)bh * N * D;
    const uint16_t* kh = k + head_off;
    const uint16_t* vh = v + head_off;
    const float sc = scale * kLog2e;

    // ---- this wave's K and V rows as B operands (lane: key column, 8 head-dim elements)
    i32x4 kreg[KS], vreg[KS];
    const int my_key = key0 + wave * 32 + col;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        i32x4 z = {0, 0, 0, 0};
        kreg[ks] = my_key < N ? *reinterpret_cast<const i32x4*>(kh + (size_t)my_key * D + ks * 16 + half * 8) : z;
        vreg[ks] = my_key < N ? *reinterpret_cast<const i32x4*>(vh + (size_t)my_key * D + ks * 16 + half * 8) : z;
    }
    // The kernel needs more than 256 registers per lane, so part of them live in the accumulation
    // half of the register file, which only MFMA can address directly.  K_j / V_j operands and the
    // dK / dV accumulators are touched by MFMA alone and live there; the score tiles, which the
    // exponentials read, are kept in ordinary registers (VACC below).
    if constexpr (D >= 128) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+a"(kreg[ks]), "+a"(vreg[ks]));
    }

    f32x16 dkacc[DT], dvacc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            dkacc[dt][r] = 0.f;
            dvacc[dt][r] = 0.f;
        }

    const int n_qtiles = (N + BQ - 1) / BQ;
    const int it0 = CAUSAL ? key0 / BQ : 0;  // first query tile that can see this key block
    const int tr_row = (lane & 15) >> 2;
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    // Masked query tiles come first: every tile when the key block is ragged (keys past N), else
    // the tiles on the causal diagonal.  They get a loop of their own so that the main loop has a
    // single straight-line body.
    const int it_masked_end = key0 + BK > N ? n_qtiles : (CAUSAL ? min(n_qtiles, (key0 + BK - 1) / BQ + 1) : it0);

    // Every query head of the group adds into the same dK_j, dV_j (grouped-query attention: the
    // gradient of a shared key/value head is the sum over the query heads that read it).
#pragma nounroll
    for (int g = 0; g < kv_group; ++g) {
    const size_t qhead = (size_t)bh * kv_group + g;
    const uint16_t* qh = q + qhead * N * D;
    const uint16_t* doh = dout + qhead * N * D;
    const float* lh = lse + qhead * N;
    const float* dh = dvec + qhead * N;

    // Q_i and dO_i tiles are contiguous runs of the row-major tensors; rows past N lie outside the
    // buffer resources and read as zero.
    const __amdgpu_buffer_rsrc_t q_rsrc = make_buffer(qh, (uint32_t)N * D * 2);
    const __amdgpu_buffer_rsrc_t do_rsrc = make_buffer(doh, (uint32_t)N * D * 2);
    // At d = 256 the staging registers of a whole tile pair (64 per lane) would not fit beside the
    // operands and accumulators: the tile travels in two halves, the first stored to LDS between
    // the two GEMM pairs of the iteration, the second at its end.
    constexpr int NG = QCH >= 8 ? 2 : 1;
    constexpr int QG = QCH / NG;
    i32x4 qpre[QG], dopre[QG];
    float lpre = 0.f;  // threads 0..63 carry L, 64..127 carry D
    int lrow = 0;
    // The next tile travels global -> registers (issued at the top of an iteration) -> LDS (at its
    // end).  Spreading the loads and the LDS writes over the MFMA steps was measured and is no
    // faster: the single wave of a SIMD is bound by its own instruction issue, not by where in
    // the iteration an instruction sits.
    auto load_group = [&](int it, int grp) {  // chunks grp * QG .. of the Q_i and dO_i tiles
#pragma unroll
        for (int j = 0; j < QG; ++j) {
            const int i = grp * QG + j;
            qpre[j] = buffer_load_16B(q_rsrc, it * BQ * D * 2 + (tid + i * NT) * 16);
            dopre[j] = buffer_load_16B(do_rsrc, it * BQ * D * 2 + (tid + i * NT) * 16);
        }
    };
    auto load_ld = [&](int it) {
        if (tid < 2 * BQ) {
            // the raw value only: anything computed from it here would make the wave wait for the
            // load on the spot, once per iteration
            lrow = it * BQ + (tid & (BQ - 1));
            lpre = (tid < BQ ? lh : dh)[min(lrow, N - 1)];
        }
    };
    auto store_group = [&](int st, int grp) {
#pragma unroll
        for (int j = 0; j < QG; ++j) {
            int c = tid + (grp * QG + j) * NT;
            int row = c / CPR, cc = c % CPR;
            *reinterpret_cast<i32x4*>(lds_t[st] + row * RSTR + cc * 8) = qpre[j];
            *reinterpret_cast<i32x4*>(lds_t[2 + st] + row * RSTR + cc * 8) = dopre[j];
        }
    };
    auto store_ld = [&](int st) {
        // rows past N get L = +inf so that P = exp2(0 - inf) = 0, and D = 0.  D is kept negated:
        // the dP accumulators start from -D_i, so dP - D comes out of the MFMAs
        if (tid < BQ) lds_l[st][tid] = lrow < N ? lpre * kLog2e : INFINITY;
        else if (tid < 2 * BQ) lds_d[st][tid - BQ] = lrow < N ? -lpre : 0.f;
    };

    if (it0 < n_qtiles) {
        load_ld(it0);
#pragma unroll
        for (int grp = 0; grp < NG; ++grp) {
            load_group(it0, grp);
            store_group(0, grp);
        }
        store_ld(0);
    }
    __syncthreads();

    auto iteration = [&](int it, auto mask_tag) {
        const int st = (it - it0) & 1;
        const int q0 = it * BQ;
        const bool more = it + 1 < n_qtiles;
        if (more) {
            load_group(it + 1, 0);
            load_ld(it + 1);
        }

        // One wave per SIMD: nothing but this wave's own instruction stream can keep the matrix
        // pipe busy while the exponentials run.  The iteration is therefore software-pipelined by
        // hand over its two 32-query sub-tiles (the intra-warpgroup overlap of the paper's
        // Algorithm 2, applied to the backward pass):
        //   stage 1: S, dP of sub-tile 0                      (MFMA only)
        //   stage 2: S, dP of sub-tile 1  ||  P, dS of sub-tile 0
        //   stage 3: dV, dK += sub-tile 0 ||  P, dS of sub-tile 1
        //   stage 4: dV, dK += sub-tile 1                     (MFMA only)
        // Every step ends in a full scheduling barrier so the interleaving below is what runs, and
        // LDS operand reads lead their MFMAs by KP steps.
        auto body = [&](auto mask_tag) {
            constexpr bool MASK = decltype(mask_tag)::value;
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            i32x4 pa[2][2], dsa[2][2];  // [sub-tile][16-query slab]: P^T and dS^T as A operands
            f32x16 sacc[2], pacc[2];

            // This tile's LDS addresses, one register each; every read below adds a compile-time
            // offset that fits the instruction's immediate field.
            // Row reads: lane (col, half) takes 8 elements from 16 ks + 8 half of row col (+ 32 per
            // sub-tile).  Transposing reads: lane takes 4 elements at tr_col of row 4 half + tr_row
            // (+ 8 for the second read, + 16 per slab), 32 elements further per d-tile.
            uint32_t q_rows = lds_address(lds_t[st]) + (col * RSTR + half * 8) * 2;
            uint32_t q_tr = lds_address(lds_t[st]) + ((4 * half + tr_row) * RSTR + tr_col + col0) * 2;
            uint32_t l_rows = lds_address(lds_l[st]) + 16 * half;  // 4 consecutive rows from 4 * half
            uint32_t d_rows = lds_address(lds_d[st]) + 16 * half;
            asm volatile("" : "+v"(q_rows), "+v"(q_tr), "+v"(l_rows), "+v"(d_rows));
            auto row_addr = [&](int u) -> uint32_t {  // step u = (sub-tile, ks) of stages 1 and 2
                const int sub = u / KS, ks = u % KS;
                return q_rows + (sub * 32 * RSTR + ks * 16) * 2;
            };
            auto tr_addr = [&](int u, int hi) -> uint32_t {  // step u = (16-query slab, d-tile) of stages 3 and 4
                const int slab = u / DT, dt = u % DT;
                return q_tr + ((slab * 16 + hi * 8) * RSTR + dt * 32) * 2;
            };

            // L (log2 units) of the lane's query rows, fetched four rows at a time one step before
            // they are needed so that few of them are live at once
            f32x4 l4[2][4];
            auto fetch_l = [&](int sub, int g) { l4[sub][g] = lds_load_4f(l_rows + (sub * 32 + 8 * g) * 4); };
            // dP starts from -D_i: accumulator registers 4g..4g+3 are query rows 8g+4*half..+3
            auto init_dp = [&](int sub) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 t = lds_load_4f(d_rows + (sub * 32 + 8 * g) * 4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) pacc[sub][4 * g + r] = t[r];
                }
            };

            // elements 2c, 2c+1 of a sub-tile: P, dS and one packed register of each.  The two elements
            // are computed in the shadows of two different MFMAs (softmax_elem after each), the pair
            // is packed after the second.
            float pv[8][2], dsv[8][2];  // indexed by the pair's number within its sub-tile
            auto softmax_elem = [&](int sub, int c, int e) {
                const int rr = 2 * c + e, g = rr >> 2, r = rr & 3;
                float p = fast_exp2(__builtin_fmaf(sacc[sub][rr], sc, -l4[sub][g][r]));
                if constexpr (MASK) {
                    const int qi = q0 + sub * 32 + 8 * g + 4 * half + r;
                    const bool masked = my_key >= N || (CAUSAL && my_key > qi);
                    p = masked ? 0.f : p;
                }
                pv[c][e] = p;
                dsv[c][e] = p * pacc[sub][rr];
            };
            auto softmax_pack = [&](int sub, int c) {
                pa[sub][c >> 2][c & 3] = E::pack2(pv[c][0], pv[c][1]);
                dsa[sub][c >> 2][c & 3] = E::pack2(dsv[c][0], dsv[c][1]);
            };

            // ---- stages 1 and 2: S = Q_i K_j^T, dP = dO_i V_j^T
            {
                constexpr int NU = 2 * KS;
                i32x4 aq[KP], ado[KP];
#pragma unroll
                for (int u = 0; u < KP; ++u) {
                    aq[u] = lds_load_16B(row_addr(u));
                    ado[u] = lds_load_16B(row_addr(u) + DO_DIST);
                }
                init_dp(0);
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int sub = u / KS, ks = u % KS;
                    i32x4 a0 = aq[u % KP], a1 = ado[u % KP];
                    if (u + KP < NU) {
                        aq[u % KP] = lds_load_16B(row_addr(u + KP));
                        ado[u % KP] = lds_load_16B(row_addr(u + KP) + DO_DIST);
                    }
                    if (u == KS - 2) init_dp(1);
                    // A wave issues in order and its second MFMA waits for the matrix pipe to take it:
                    // vector work placed after both MFMAs of a step runs in the shadow of the second
                    // one only.  Half of it goes between the two.
                    if constexpr (VACC) {
                        if (ks == 0) MfmaVgprAcc<Tag>::first(sacc[sub], a0, kreg[ks]);
                        else MfmaVgprAcc<Tag>::run(sacc[sub], a0, kreg[ks]);
                    } else {
                        sacc[sub] = E::mma(a0, kreg[ks], ks == 0 ? zero : sacc[sub]);
                    }
                    if (sub == 1) {
                        // sub-tile 0's results were written by MFMAs the hazard checker cannot see
                        if constexpr (VACC) {
                            if (ks == 0) mfma_result_wait(sacc[0], pacc[0]);
                        }
                        // the 8 register pairs of sub-tile 0 spread over the KS steps (pair c runs at
                        // step c KS / 8); the L group of a pair is fetched one step before the step
                        // that needs it first
#pragma unroll
                        for (int g = 1; g < 4; ++g)
                            if ((2 * g * KS) / 8 == ks + 1) fetch_l(0, g);
                        if (ks == KS - 1) fetch_l(1, 0);
#pragma unroll
                        for (int c = 0; c < 8; ++c)
                            if ((c * KS) / 8 == ks) softmax_elem(0, c, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if constexpr (VACC) MfmaVgprAcc<Tag>::run(pacc[sub], a1, vreg[ks]);
                    else pacc[sub] = E::mma(a1, vreg[ks], pacc[sub]);
                    if (sub == 0 && ks == KS - 1) fetch_l(0, 0);
                    if (sub == 1) {
#pragma unroll
                        for (int c = 0; c < 8; ++c)
                            if ((c * KS) / 8 == ks) {
                                softmax_elem(0, c, 1);
                                softmax_pack(0, c);
                            }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }

            if constexpr (NG == 2) {
                if (more) {  // the other LDS buffers are free for the whole iteration
                    store_group(st ^ 1, 0);
                    load_group(it + 1, 1);
                }
            }

            // ---- stages 3 and 4: dV_j += P^T dO_i, dK_j += dS^T Q_i (contract over the tile's queries)
            {
                constexpr int NU = 2 * 2 * DT;  // (sub, slab, d-tile)
                i32x2 dlo[KP], dhi[KP], qlo[KP], qhi[KP];
#pragma unroll
                for (int u = 0; u < KP; ++u) {
                    dlo[u] = lds_read_tr16(tr_addr(u, 0) + DO_DIST);
                    dhi[u] = lds_read_tr16(tr_addr(u, 1) + DO_DIST);
                    qlo[u] = lds_read_tr16(tr_addr(u, 0));
                    qhi[u] = lds_read_tr16(tr_addr(u, 1));
                }
#pragma unroll
                for (int u = 0; u < NU; ++u) {
                    const int sub = u / (2 * DT), s2 = (u / DT) % 2, dt = u % DT;
                    const int w = u % KP;
                    i32x4 b = {dlo[w][0], dlo[w][1], dhi[w][0], dhi[w][1]};
                    i32x4 b2 = {qlo[w][0], qlo[w][1], qhi[w][0], qhi[w][1]};
                    if (u + KP < NU) {
                        dlo[w] = lds_read_tr16(tr_addr(u + KP, 0) + DO_DIST);
                        dhi[w] = lds_read_tr16(tr_addr(u + KP, 1) + DO_DIST);
                        qlo[w] = lds_read_tr16(tr_addr(u + KP, 0));
                        qhi[w] = lds_read_tr16(tr_addr(u + KP, 1));
                    }
                    dvacc[dt] = E::mma(pa[sub][s2], b, dvacc[dt]);
                    constexpr int PP = 8 / (2 * DT);
                    if (sub == 0) {
                        if constexpr (VACC) {
                            if (u == 0) mfma_result_wait(sacc[1], pacc[1]);
                        }
#pragma unroll
                        for (int g = 1; g < 4; ++g)
                            if ((2 * g) / PP == u + 1) fetch_l(1, g);
#pragma unroll
                        for (int p = 0; p < PP; ++p) softmax_elem(1, u * PP + p, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    dkacc[dt] = E::mma(dsa[sub][s2], b2, dkacc[dt]);
                    if (sub == 0) {
#pragma unroll
                        for (int p = 0; p < PP; ++p) {
                            softmax_elem(1, u * PP + p, 1);
                            softmax_pack(1, u * PP + p);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        body(mask_tag);

        if (more) {
            store_group(st ^ 1, NG - 1);
            store_ld(st ^ 1);
        }
        __syncthreads();
    };
    int it = it0;
    for (; it < it_masked_end; ++it) iteration(it, std::true_type{});
    for (; it < n_qtiles; ++it) iteration(it, std::false_type{});
    }  // query heads of the group

    // ---- epilogue: dK_j = scale * acc, dV_j = acc  (rows = keys 8g+4h+r of this wave, col = d)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int key = key0 + wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key < N) {
                size_t off = head_off + (size_t)key * D + col0 + dt * 32 + col;
                dk[off] = (uint16_t)(E::pack2(dkacc[dt][r] * scale, 0.f) & 0xFFFF);
                dv[off] = (uint16_t)(E::pack2(dvacc[dt][r], 0.f) & 0xFFFF);
            }
        }
}

// ---------------------------------------------------------------------------------------
// dQ pass: the forward kernel's structure with dO alongside Q and K^T in place of V^T.
template <typename Tag, int D, int BC, int NW, bool CAUSAL>
__global__ void __launch_bounds__(NW * 64, NW == 8 ? 2 : 1)
fa_bwd_dq_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                 const uint16_t* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ dvec,
                 uint16_t* __restrict__ dq, int N, int n_qtiles, int total_wg, int kv_group, float scale) {
    [[maybe_unused]] ClockSpan clock_span;  // measurement builds only; empty otherwise
    constexpr int NT = NW * 64;
    constexpr int BR = NW * 32;
    constexpr int RSTR = bwd_row_stride(D);  // K tile: row reads and transposed reads
    constexpr int VSTR = D + 8;              // V tile: row reads only
    constexpr int KT = BC / 32;
    constexpr int KS = D / 16;
    constexpr int DT = D / 32;
    constexpr int SL = BC / 16;
    constexpr int CPR = D / 8;
    constexpr int CPT = BC * CPR / NT;
    static_assert((BC * CPR) % NT == 0, "tile must divide evenly over the workgroup");
    using E = Elem<Tag>;

    __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][BC * RSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_v[2][BC * VSTR];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int bh = id / n_qtiles;
    int qt = id % n_qtiles;
    if (CAUSAL) qt = n_qtiles - 1 - qt;  // longest rows first

    const size_t head_off = (size_t)bh * N * D;
    const size_t kv_off = (size_t)(bh / kv_group) * N * D;  // grouped-query: kv_group query heads per K/V head
    const uint16_t* kh = k + kv_off;
    const uint16_t* vh = v + kv_off;
    const int wave_q0 = qt * BR + wave * 32;
    const int qi = wave_q0 + col;
    const int qrow = min(qi, N - 1);  // rows past N compute a copy of row N-1, never stored
    const float sc = scale * kLog2e;

    i32x4 qreg[KS], doreg[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        qreg[ks] = *reinterpret_cast<const i32x4*>(q + head_off + (size_t)qrow * D + ks * 16 + half * 8);
        doreg[ks] = *reinterpret_cast<const i32x4*>(dout + head_off + (size_t)qrow * D + ks * 16 + half * 8);
    }
    const float l2 = lse[(size_t)bh * N + qrow] * kLog2e;
    const float dq_row = dvec[(size_t)bh * N + qrow];
    constexpr bool NEG_D_START = D == 64;
    f32x16 negd;
#pragma unroll
    for (int r = 0; r < 16; ++r) negd[r] = -dq_row;

    f32x16 acc[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;

    int last_q = min(qt * BR + BR, N) - 1;
    int n_blocks = CAUSAL ? (last_q / BC + 1) : ((N + BC - 1) / BC);

    const __amdgpu_buffer_rsrc_t k_rsrc = make_buffer(kh, (uint32_t)N * D * 2);
    const __amdgpu_buffer_rsrc_t v_rsrc = make_buffer(vh, (uint32_t)N * D * 2);
    i32x4 kpre[CPT], vpre[CPT];
    auto load_tile = [&](int key0) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            kpre[i] = buffer_load_16B(k_rsrc, key0 * D * 2 + (tid + i * NT) * 16);
            vpre[i] = buffer_load_16B(v_rsrc, key0 * D * 2 + (tid + i * NT) * 16);
        }
    };
    auto store_tile = [&](int st) {
#pragma unroll
        for (int i = 0; i < CPT; ++i) {
            int c = tid + i * NT;
            int row = c / CPR, cc = c % CPR;
            *reinterpret_cast<i32x4*>(lds_k[st] + row * RSTR + cc * 8) = kpre[i];
            *reinterpret_cast<i32x4*>(lds_v[st] + row * VSTR + cc * 8) = vpre[i];
        }
    };
    load_tile(0);
    store_tile(0);
    // One wave per SIMD (d = 256): the kernel may use more than 256 registers per lane, MFMA results
    // then land in the accumulation half of the register file, and the score tiles would pay a copy per
    // element on their way to the exponentials.  They are produced by MfmaVgprAcc into ordinary
    // registers instead (Q_i, dO_i, touched by MFMA alone, go to the accumulation half), and the next
    // block's K and V travel in 16-byte chunks spread over the MFMA steps: as one burst, the 16 loads
    // of a wave keep it in its own issue for over a thousand cycles (see fa_fwd_d256_kernel).
    constexpr bool ONE_WAVE = NW == 4;
    constexpr int NSTEP = KS * KT;  // MFMA steps of either GEMM group; a staging chunk every CH_EVERY of them
    constexpr int CH_EVERY = ONE_WAVE ? NSTEP / CPT : 1;
    static_assert(!ONE_WAVE || (CPT * CH_EVERY == NSTEP && SL * DT == NSTEP), "chunks must spread evenly");
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {  // loads done before the loop
        if constexpr (ONE_WAVE) asm volatile("" : "+a"(qreg[ks]), "+a"(doreg[ks]));
        else asm volatile("" : "+v"(qreg[ks]), "+v"(doreg[ks]));
    }
    __syncthreads();

    const int tr_row = (lane & 15) >> 2;
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    for (int t = 0; t < n_blocks; ++t) {
        const int st = t & 1;
        const int key0 = t * BC;
        const bool more = (t + 1 < n_blocks);
        // a wave whose queries all precede this block has nothing to add (causal).  With one wave per SIMD every
        // wave works every block (a fully masked one adds zeros): the branch around the interleaved staging
        // costs that instantiation a hundred registers.
        const bool wave_active = !CAUSAL || ONE_WAVE || key0 <= wave_q0 + 31;
        if (more && !(ONE_WAVE && wave_active)) load_tile(key0 + BC);

        if (wave_active) {
            // ---- S^T = K_j Q_i^T and dP^T = V_j dO_i^T
            f32x16 sacc[KT], pacc[KT];
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            const int kbase = col * RSTR + half * 8, vbase = col * VSTR + half * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int kt = 0; kt < KT; ++kt) {
                    i32x4 ak = *reinterpret_cast<const i32x4*>(lds_k[st] + kbase + kt * 32 * RSTR + ks * 16);
                    i32x4 av = *reinterpret_cast<const i32x4*>(lds_v[st] + vbase + kt * 32 * VSTR + ks * 16);
                    if constexpr (ONE_WAVE) {
                        if (ks == 0) {
                            MfmaVgprAcc<Tag>::first(sacc[kt], ak, qreg[ks]);
                            MfmaVgprAcc<Tag>::first(pacc[kt], av, doreg[ks]);
                        } else {
                            MfmaVgprAcc<Tag>::run(sacc[kt], ak, qreg[ks]);
                            MfmaVgprAcc<Tag>::run(pacc[kt], av, doreg[ks]);
                        }
                        const int u = ks * KT + kt;
                        if (more && u % CH_EVERY == 0) {
                            const int i = u / CH_EVERY;
                            kpre[i] = buffer_load_16B(k_rsrc, (key0 + BC) * D * 2 + (tid + i * NT) * 16);
                            vpre[i] = buffer_load_16B(v_rsrc, (key0 + BC) * D * 2 + (tid + i * NT) * 16);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    } else {
                        sacc[kt] = E::mma(ak, qreg[ks], ks == 0 ? zero : sacc[kt]);
                        // where registers allow, dP starts from -D (a lane owns one query, so D is one value per
                        // lane, kept as a 16-register constant): dP - D comes out of the MFMAs
                        pacc[kt] = E::mma(av, doreg[ks], ks == 0 ? (NEG_D_START ? negd : zero) : pacc[kt]);
                    }
                }
            if constexpr (ONE_WAVE) {  // results of MFMAs the hazard checker cannot see
                static_assert(!ONE_WAVE || KT == 2, "two score tiles per GEMM");
                mfma_result_wait(sacc[0], sacc[1]);
                mfma_result_wait(pacc[0], pacc[1]);
            }

            // ---- P = exp(S - L), dS = P o (dP - D), packed as the B operand of the dQ product
            // keys past N, and keys after the query when causal, get S = -inf (P = 0): one uniform branch per
            // block, not a select per element in every block
            constexpr bool MASK_BRANCH = true;
            const bool need_mask = (key0 + BC > N) || (CAUSAL && key0 + BC - 1 > wave_q0);
            const int limit = CAUSAL ? min(qi, N - 1) : N - 1;  // last visible key
            if (MASK_BRANCH && need_mask) {
                // compile-time key offsets against one per-lane bound (kept opaque: the compiler otherwise
                // hoists 32 per-element key indices out of the block loop into registers of their own)
                int bound = limit - key0 - 4 * half;
                asm volatile("" : "+v"(bound));
#pragma unroll
                for (int kt = 0; kt < KT; ++kt)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        if (kt * 32 + 8 * (r >> 2) + (r & 3) > bound) sacc[kt][r] = -INFINITY;
            }
            i32x4 dsb[SL];
#pragma unroll
            for (int kt = 0; kt < KT; ++kt) {
                float ds[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    float p = fast_exp2(__builtin_fmaf(sacc[kt][r], sc, -l2));
                    if (!MASK_BRANCH && need_mask) {
                        const int key = key0 + kt * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                        p = key > limit ? 0.f : p;
                    }
                    ds[r] = NEG_D_START ? p * pacc[kt][r] : p * (pacc[kt][r] - dq_row);
                }
#pragma unroll
                for (int s2 = 0; s2 < 2; ++s2) {
                    i32x4 w;
#pragma unroll
                    for (int e = 0; e < 4; ++e) w[e] = E::pack2(ds[8 * s2 + 2 * e], ds[8 * s2 + 2 * e + 1]);
                    dsb[2 * kt + s2] = w;
                }
            }

            // ---- dQ_i^T += K_j^T dS^T
            const uint16_t* kt_base = lds_k[st] + (4 * half + tr_row) * RSTR + tr_col;
#pragma unroll
            for (int sl = 0; sl < SL; ++sl)
#pragma unroll
                for (int dt = 0; dt < DT; ++dt) {
                    const uint16_t* p0 = kt_base + (sl * 16) * RSTR + dt * 32;
                    i32x2 lo = lds_read_tr16(p0);
                    i32x2 hi = lds_read_tr16(p0 + 8 * RSTR);
                    i32x4 a = {lo[0], lo[1], hi[0], hi[1]};
                    acc[dt] = E::mma(a, dsb[sl], acc[dt]);
                    if constexpr (ONE_WAVE) {
                        const int u = sl * DT + dt;
                        if (more && u % CH_EVERY == 0) {  // the chunks loaded beside the first GEMM group go to the other buffers
                            const int c = tid + (u / CH_EVERY) * NT;
                            *reinterpret_cast<i32x4*>(lds_k[st ^ 1] + (c / CPR) * RSTR + (c % CPR) * 8) = kpre[u / CH_EVERY];
                            *reinterpret_cast<i32x4*>(lds_v[st ^ 1] + (c / CPR) * VSTR + (c % CPR) * 8) = vpre[u / CH_EVERY];
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
        }

        if (more && !(ONE_WAVE && wave_active)) store_tile(st ^ 1);
        __syncthreads();
    }

    // dQ_i = scale * acc.  Every LDS read of the loop was followed by a barrier, so the K and V
    // buffers are free: each wave takes 4 KiB of them to transpose its tile into whole 128-byte lines.
    static_assert(NW <= 8 && sizeof(lds_k) >= 4 * 4096 && sizeof(lds_v) >= 4 * 4096, "patches must fit");
    char* patch = (wave < 4 ? reinterpret_cast<char*>(&lds_k[0][0]) : reinterpret_cast<char*>(&lds_v[0][0])) +
                  (wave & 3) * 4096;
    store_rows_via_lds<Tag, DT>(acc, scale, patch, make_buffer(dq + head_off, (uint32_t)N * D * 2), wave_q0, lane);
}

// ---------------------------------------------------------------------------------------
size_t bwd_workspace_bytes(int B, int H, int N, int d) {
    (void)d;
    size_t rows = (size_t)B * H * N;
    return (rows * sizeof(float) + 15) & ~(size_t)15;  // D = rowsum(dO o O)
}

template <typename Tag, int D>
static int launch_bwd_t(const void* q, const void* k, const void* v, const void* o, const float* lse,
                        const void* dout, void* dq, void* dk, void* dv, void* workspace, int B, int H, int H_kv,
                        int N, float scale, int causal, hipStream_t stream) {
    const long rows = (long)B * H * N;
    float* dvec = static_cast<float*>(workspace);
    auto u16 = [](const void* p) { return static_cast<const uint16_t*>(p); };
    // every size check comes before the first launch: a call that fails has enqueued nothing
    const int n_kblocks = (N + 127) / 128;
    const long total = (long)B * H_kv * n_kblocks;
    constexpr int BC = 64, NW = D == 256 ? 4 : 8;  // d = 256: a wave needs the whole register file
    const int n_qtiles = (N + NW * 32 - 1) / (NW * 32);
    const long total_q = (long)B * H * n_qtiles;
    if (total > 0x7fffffffL || total_q > 0x7fffffffL) return FA_ERR_SHAPE;

    constexpr int kRowsPerWg = 256 / (D / 8);
    hipLaunchKernelGGL((fa_bwd_preprocess_kernel<Tag, D>), dim3((unsigned)((rows + kRowsPerWg - 1) / kRowsPerWg)),
                       dim3(256), 0, stream,
                       u16(o), u16(dout), dvec, rows);
    if (hipGetLastError() != hipSuccess) return FA_ERR_LAUNCH;

    const dim3 kv_grid((unsigned)total, D > 128 ? D / 128 : 1);  // y: 128-column slices of dK, dV
    if (causal)
        hipLaunchKernelGGL((fa_bwd_dkdv_kernel<Tag, D, true>), kv_grid, dim3(256), 0, stream, u16(q),
                           u16(k), u16(v), u16(dout), lse, dvec, static_cast<uint16_t*>(dk),
                           static_cast<uint16_t*>(dv), N, n_kblocks, (int)total, H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_bwd_dkdv_kernel<Tag, D, false>), kv_grid, dim3(256), 0, stream, u16(q),
                           u16(k), u16(v), u16(dout), lse, dvec, static_cast<uint16_t*>(dk),
                           static_cast<uint16_t*>(dv), N, n_kblocks, (int)total, H / H_kv, scale);
    if (hipGetLastError() != hipSuccess) return FA_ERR_LAUNCH;

    if (causal)
        hipLaunchKernelGGL((fa_bwd_dq_kernel<Tag, D, BC, NW, true>), dim3((unsigned)total_q), dim3(NW * 64), 0, stream,
                           u16(q), u16(k), u16(v), u16(dout), lse, dvec, static_cast<uint16_t*>(dq), N, n_qtiles,
                           (int)total_q, H / H_kv, scale);
    else
        hipLaunchKernelGGL((fa_bwd_dq_kernel<Tag, D, BC, NW, false>), dim3((unsigned)total_q), dim3(NW * 64), 0, stream,
                           u16(q), u16(k), u16(v), u16(dout), lse, dvec, static_cast<uint16_t*>(dq), N, n_qtiles,
                           (int)total_q, H / H_kv, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

int launch_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
               void* dq, void* dk, void* dv, void* workspace, int B, int H, int H_kv, int N, int d, float scale,
               int causal, int dtype, hipStream_t stream) {
#define FA_BWD_CASE(TAG, DD) \
    return launch_bwd_t<TAG, DD>(q, k, v, o, lse, dout, dq, dk, dv, workspace, B, H, H_kv, N, scale, causal, stream)
    if (dtype == FA_BF16 && d == 128) FA_BWD_CASE(bf16_tag, 128);
    if (dtype == FA_BF16 && d == 64) FA_BWD_CASE(bf16_tag, 64);
    if (dtype == FA_F16 && d == 128) FA_BWD_CASE(f16_tag, 128);
    if (dtype == FA_F16 && d == 64) FA_BWD_CASE(f16_tag, 64);
    if (dtype == FA_BF16 && d == 256) FA_BWD_CASE(bf16_tag, 256);
    if (dtype == FA_F16 && d == 256) FA_BWD_CASE(f16_tag, 256);
#undef FA_BWD_CASE
    return FA_ERR_UNSUPPORTED;
}

}  // namespace fa

FA_CLOCK_SPAN_READER(fa_debug_clock_span_bwd)
