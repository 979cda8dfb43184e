// Backward attention for gfx950, head dimension 128, bf16 / fp16 (paper Algorithm 3).
//
//   preprocess : D = rowsum(dO o O) per query row, and the fp32 dQ accumulator is cleared
//   main       : one workgroup per block of 128 keys (wave w owns keys 32w..32w+31); loop over
//                tiles of 64 queries:  S = Q_i K_j^T,  dP = dO_i V_j^T,  P = exp(S - L),
//                dS = P o (dP - D),  dV_j += P^T dO_i,  dK_j += dS^T Q_i  (on chip),
//                dQ_i += dS K_j  (fp32 atomics into the accumulator, as in the paper)
//   convert    : dQ = scale * accumulator, cast to the I/O dtype
//
// Register layouts: S and dP are computed with queries as MFMA rows and keys as columns, so a
// lane owns one key and 16 queries in its accumulator registers; packed to 16 bits those
// registers are directly the A operand (keys x queries) of the dV and dK products, whose B
// operands (dO, Q as queries x d) come from transposing LDS reads.  dQ contracts over keys,
// which lanes do not own, so dS^T goes through LDS once (written [key][query], read back with
// transposing reads) -- the role the dQ staging buffer and writer warp play in Algorithm 3.
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

#include "fa_device.h"
#include "fa_launch.h"

namespace fa {

constexpr int kBwdD = 128;
constexpr int kPipe = 4;  // MFMA steps by which LDS operand reads lead their use

// ---------------------------------------------------------------------------------------
template <typename Tag>
__global__ void __launch_bounds__(256)
fa_bwd_preprocess_kernel(const uint16_t* __restrict__ o, const uint16_t* __restrict__ dout,
                         float* __restrict__ dvec, float* __restrict__ dq_acc, long rows) {
    constexpr int D = kBwdD;
    using E = Elem<Tag>;
    const int lane16 = threadIdx.x & 15;
    long row = (long)blockIdx.x * 16 + (threadIdx.x >> 4);
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
        f32x4 z = {0.f, 0.f, 0.f, 0.f};
        *reinterpret_cast<f32x4*>(dq_acc + row * D + lane16 * 8) = z;
        *reinterpret_cast<f32x4*>(dq_acc + row * D + lane16 * 8 + 4) = z;
    }
#pragma unroll
    for (int off = 8; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
    if (row < rows && lane16 == 0) dvec[row] = acc;
}

template <typename Tag>
__global__ void __launch_bounds__(256)
fa_bwd_convert_dq_kernel(const float* __restrict__ dq_acc, uint16_t* __restrict__ dq, long n8, float scale) {
    using E = Elem<Tag>;
    long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    f32x4 a = *reinterpret_cast<const f32x4*>(dq_acc + i * 8);
    f32x4 b = *reinterpret_cast<const f32x4*>(dq_acc + i * 8 + 4);
    i32x4 w = {E::pack2(a[0] * scale, a[1] * scale), E::pack2(a[2] * scale, a[3] * scale),
               E::pack2(b[0] * scale, b[1] * scale), E::pack2(b[2] * scale, b[3] * scale)};
    *reinterpret_cast<i32x4*>(dq + i * 8) = w;
}

// ---------------------------------------------------------------------------------------
template <typename Tag, bool CAUSAL>
__global__ void __launch_bounds__(256, 1)
fa_bwd_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
              const uint16_t* __restrict__ dout, const float* __restrict__ lse, const float* __restrict__ dvec,
              float* __restrict__ dq_acc, uint16_t* __restrict__ dk, uint16_t* __restrict__ dv, int N,
              int n_kblocks, int total_wg, float scale) {
    constexpr int D = kBwdD;
    constexpr int BK = 128;        // keys per workgroup
    constexpr int BQ = 64;         // queries per loop iteration
    constexpr int NT = 256;
    constexpr int RSTR = D + 8;    // row stride (elements) of the Q, dO and K tiles
    constexpr int SSTR = BQ + 8;   // row stride of the dS^T tile [key][query]
    constexpr int KS = D / 16;
    constexpr int DT = D / 32;
    constexpr int CPR = D / 8;     // 16-byte chunks per row
    constexpr int QCH = BQ * CPR / NT;  // chunks per thread for a Q / dO tile
    constexpr int KCH = BK * CPR / NT;
    using E = Elem<Tag>;

    __shared__ __attribute__((aligned(16))) uint16_t lds_q[2][BQ * RSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_do[2][BQ * RSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_k[BK * RSTR];
    __shared__ __attribute__((aligned(16))) uint16_t lds_ds[BK * SSTR];
    __shared__ __attribute__((aligned(16))) float lds_l[2][BQ];
    __shared__ __attribute__((aligned(16))) float lds_d[2][BQ];

    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63;
    const int col = lane & 31, half = lane >> 5;

    int id = xcd_contiguous(blockIdx.x, total_wg);
    const int bh = id / n_kblocks;
    const int kb = id % n_kblocks;  // causal: key block 0 has the longest loop and comes first
    const int key0 = kb * BK;

    const size_t head_off = (size_t)bh * N * D;
    const uint16_t* qh = q + head_off;
    const uint16_t* kh = k + head_off;
    const uint16_t* vh = v + head_off;
    const uint16_t* doh = dout + head_off;
    const float* lh = lse + (size_t)bh * N;
    const float* dh = dvec + (size_t)bh * N;
    float* dqh = dq_acc + head_off;
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
    // ---- the whole K block in LDS for the dQ product
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
        int c = tid + i * NT;
        int row = c / CPR, cc = c % CPR;
        i32x4 z = {0, 0, 0, 0};
        i32x4 w = key0 + row < N ? *reinterpret_cast<const i32x4*>(kh + (size_t)(key0 + row) * D + cc * 8) : z;
        *reinterpret_cast<i32x4*>(lds_k + row * RSTR + cc * 8) = w;
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

    // Q_i and dO_i tiles are contiguous runs of the row-major tensors; rows past N lie outside the
    // buffer resources and read as zero.
    const __amdgpu_buffer_rsrc_t q_rsrc = make_buffer(qh, (uint32_t)N * D * 2);
    const __amdgpu_buffer_rsrc_t do_rsrc = make_buffer(doh, (uint32_t)N * D * 2);
    i32x4 qpre[QCH], dopre[QCH];
    float lpre = 0.f;  // threads 0..63 carry L, 64..127 carry D
    auto load_tile = [&](int it) {
        const int q0 = it * BQ;
#pragma unroll
        for (int i = 0; i < QCH; ++i) {
            qpre[i] = buffer_load_16B(q_rsrc, q0 * D * 2 + (tid + i * NT) * 16);
            dopre[i] = buffer_load_16B(do_rsrc, q0 * D * 2 + (tid + i * NT) * 16);
        }
        if (tid < 2 * BQ) {
            const int r = q0 + (tid & (BQ - 1));
            const float* src = tid < BQ ? lh : dh;
            float x = src[min(r, N - 1)];
            // rows past N get L = +inf so that P = exp2(0 - inf) = 0, and D = 0
            lpre = tid < BQ ? (r < N ? x * kLog2e : INFINITY) : (r < N ? x : 0.f);
        }
    };
    auto store_tile = [&](int st) {
#pragma unroll
        for (int i = 0; i < QCH; ++i) {
            int c = tid + i * NT;
            int row = c / CPR, cc = c % CPR;
            *reinterpret_cast<i32x4*>(lds_q[st] + row * RSTR + cc * 8) = qpre[i];
            *reinterpret_cast<i32x4*>(lds_do[st] + row * RSTR + cc * 8) = dopre[i];
        }
        if (tid < BQ) lds_l[st][tid] = lpre;
        else if (tid < 2 * BQ) lds_d[st][tid - BQ] = lpre;
    };

    if (it0 < n_qtiles) {
        load_tile(it0);
        store_tile(0);
    }
    __syncthreads();

    const int tr_row = (lane & 15) >> 2;
    const int tr_col = 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    for (int it = it0; it < n_qtiles; ++it) {
        const int st = (it - it0) & 1;
        const int q0 = it * BQ;
        const bool more = it + 1 < n_qtiles;
        if (more) load_tile(it + 1);

        i32x4 pa[2][2], dsa[2][2];  // [query sub-tile][16-query slab]: P^T and dS^T as A operands
        const bool need_mask = key0 + BK > N || (CAUSAL && key0 + BK - 1 > q0);

        // ---- S = Q_i K_j^T and dP = dO_i V_j^T for both 32-query sub-tiles.  With one wave per SIMD
        // nothing else hides LDS latency, so operand reads run kPipe steps ahead of the MFMAs.
        f32x16 sacc[2], pacc[2];
        {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            constexpr int NU = 2 * KS;
            const uint16_t* qrow = lds_q[st] + col * RSTR + half * 8;
            const uint16_t* dorow = lds_do[st] + col * RSTR + half * 8;
            i32x4 aq[kPipe], ado[kPipe];
#pragma unroll
            for (int u = 0; u < kPipe; ++u) {
                aq[u] = *reinterpret_cast<const i32x4*>(qrow + (u / KS) * 32 * RSTR + (u % KS) * 16);
                ado[u] = *reinterpret_cast<const i32x4*>(dorow + (u / KS) * 32 * RSTR + (u % KS) * 16);
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int sub = u / KS, ks = u % KS;
                i32x4 a0 = aq[u % kPipe], a1 = ado[u % kPipe];
                if (u + kPipe < NU) {
                    const int v = u + kPipe;
                    aq[u % kPipe] = *reinterpret_cast<const i32x4*>(qrow + (v / KS) * 32 * RSTR + (v % KS) * 16);
                    ado[u % kPipe] = *reinterpret_cast<const i32x4*>(dorow + (v / KS) * 32 * RSTR + (v % KS) * 16);
                }
                sacc[sub] = E::mma(a0, kreg[ks], ks == 0 ? zero : sacc[sub]);
                pacc[sub] = E::mma(a1, vreg[ks], ks == 0 ? zero : pacc[sub]);
                __builtin_amdgcn_sched_barrier(0x6);  // only VALU / SALU may move across a step
            }
        }

        // ---- P = exp(S - L), dS = P o (dP - D); pack as A operands; dS^T to LDS
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            float pv[16], dsv[16];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int ql = sub * 32 + 8 * g + 4 * half;  // first of 4 consecutive query rows
                f32x4 l4 = *reinterpret_cast<const f32x4*>(&lds_l[st][ql]);
                f32x4 d4 = *reinterpret_cast<const f32x4*>(&lds_d[st][ql]);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float p = fast_exp2(__builtin_fmaf(sacc[sub][4 * g + r], sc, -l4[r]));
                    if (need_mask) {
                        bool masked = my_key >= N || (CAUSAL && my_key > q0 + ql + r);
                        p = masked ? 0.f : p;
                    }
                    pv[4 * g + r] = p;
                    dsv[4 * g + r] = p * (pacc[sub][4 * g + r] - d4[r]);
                }
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    pa[sub][s2][e] = E::pack2(pv[8 * s2 + 2 * e], pv[8 * s2 + 2 * e + 1]);
                    dsa[sub][s2][e] = E::pack2(dsv[8 * s2 + 2 * e], dsv[8 * s2 + 2 * e + 1]);
                }
            }
            // row = this lane's key, 4 consecutive queries per group
            uint16_t* dsrow = lds_ds + (wave * 32 + col) * SSTR + sub * 32 + 4 * half;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                i32x2 w = {dsa[sub][g >> 1][2 * (g & 1)], dsa[sub][g >> 1][2 * (g & 1) + 1]};
                *reinterpret_cast<i32x2*>(dsrow + 8 * g) = w;
            }
        }

        // ---- dV_j += P^T dO_i,  dK_j += dS^T Q_i   (contract over the tile's queries)
        {
            constexpr int NU = 2 * 2 * DT;  // (sub, slab, d-tile)
            const int rbase = (4 * half + tr_row) * RSTR + tr_col;
            auto off = [&](int u) { return rbase + ((u / DT) * 16) * RSTR + (u % DT) * 32; };
            i32x2 dlo[kPipe], dhi[kPipe], qlo[kPipe], qhi[kPipe];
#pragma unroll
            for (int u = 0; u < kPipe; ++u) {
                dlo[u] = lds_read_tr16(lds_do[st] + off(u));
                dhi[u] = lds_read_tr16(lds_do[st] + off(u) + 8 * RSTR);
                qlo[u] = lds_read_tr16(lds_q[st] + off(u));
                qhi[u] = lds_read_tr16(lds_q[st] + off(u) + 8 * RSTR);
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int sub = u / (2 * DT), s2 = (u / DT) % 2, dt = u % DT;
                const int w = u % kPipe;
                i32x4 b = {dlo[w][0], dlo[w][1], dhi[w][0], dhi[w][1]};
                i32x4 b2 = {qlo[w][0], qlo[w][1], qhi[w][0], qhi[w][1]};
                if (u + kPipe < NU) {
                    dlo[w] = lds_read_tr16(lds_do[st] + off(u + kPipe));
                    dhi[w] = lds_read_tr16(lds_do[st] + off(u + kPipe) + 8 * RSTR);
                    qlo[w] = lds_read_tr16(lds_q[st] + off(u + kPipe));
                    qhi[w] = lds_read_tr16(lds_q[st] + off(u + kPipe) + 8 * RSTR);
                }
                dvacc[dt] = E::mma(pa[sub][s2], b, dvacc[dt]);
                dkacc[dt] = E::mma(dsa[sub][s2], b2, dkacc[dt]);
                __builtin_amdgcn_sched_barrier(0x6);
            }
        }

        __syncthreads();  // dS^T of all four waves is in LDS

        // ---- dQ_i += dS K_j: this wave produces head-dim columns 32w..32w+31 of both sub-tiles
        f32x16 dqacc[2];
        {
            const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            constexpr int NU = BK / 16;
            constexpr int PD = kPipe < NU ? kPipe : NU;
            const int kb0 = (4 * half + tr_row) * RSTR + wave * 32 + tr_col;
            const int sb0 = (4 * half + tr_row) * SSTR + tr_col;
            i32x2 blo[PD], bhi[PD], a0lo[PD], a0hi[PD], a1lo[PD], a1hi[PD];
            auto load = [&](int w, int s) {
                blo[w] = lds_read_tr16(lds_k + kb0 + 16 * s * RSTR);
                bhi[w] = lds_read_tr16(lds_k + kb0 + (16 * s + 8) * RSTR);
                a0lo[w] = lds_read_tr16(lds_ds + sb0 + 16 * s * SSTR);
                a0hi[w] = lds_read_tr16(lds_ds + sb0 + (16 * s + 8) * SSTR);
                a1lo[w] = lds_read_tr16(lds_ds + sb0 + 16 * s * SSTR + 32);
                a1hi[w] = lds_read_tr16(lds_ds + sb0 + (16 * s + 8) * SSTR + 32);
            };
#pragma unroll
            for (int u = 0; u < PD; ++u) load(u, u);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int w = u % PD;
                i32x4 b = {blo[w][0], blo[w][1], bhi[w][0], bhi[w][1]};
                i32x4 a0 = {a0lo[w][0], a0lo[w][1], a0hi[w][0], a0hi[w][1]};
                i32x4 a1 = {a1lo[w][0], a1lo[w][1], a1hi[w][0], a1hi[w][1]};
                if (u + PD < NU) load(w, u + PD);
                dqacc[0] = E::mma(a0, b, u == 0 ? zero : dqacc[0]);
                dqacc[1] = E::mma(a1, b, u == 0 ? zero : dqacc[1]);
                __builtin_amdgcn_sched_barrier(0x6);
            }
        }
#pragma unroll
        for (int sub = 0; sub < 2; ++sub)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int qi = q0 + sub * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
#ifdef FA_EXP_NOATOMIC
                if (qi < N && dqacc[sub][r] == 123.456f) dqh[(size_t)qi * D + wave * 32 + col] = dqacc[sub][r];
#else
                if (qi < N) unsafeAtomicAdd(dqh + (size_t)qi * D + wave * 32 + col, dqacc[sub][r]);
#endif
            }

        if (more) store_tile(st ^ 1);
        __syncthreads();
    }

    // ---- epilogue: dK_j = scale * acc, dV_j = acc  (rows = keys 8g+4h+r of this wave, col = d)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            int key = key0 + wave * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (key < N) {
                size_t off = head_off + (size_t)key * D + dt * 32 + col;
                dk[off] = (uint16_t)(E::pack2(dkacc[dt][r] * scale, 0.f) & 0xFFFF);
                dv[off] = (uint16_t)(E::pack2(dvacc[dt][r], 0.f) & 0xFFFF);
            }
        }
}

// ---------------------------------------------------------------------------------------
size_t bwd_workspace_bytes(int B, int H, int N, int d) {
    size_t rows = (size_t)B * H * N;
    return rows * d * sizeof(float) + ((rows * sizeof(float) + 15) & ~(size_t)15);
}

template <typename Tag>
static int launch_bwd_t(const void* q, const void* k, const void* v, const void* o, const float* lse,
                        const void* dout, void* dq, void* dk, void* dv, void* workspace, int B, int H, int N,
                        float scale, int causal, hipStream_t stream) {
    constexpr int D = kBwdD;
    const long rows = (long)B * H * N;
    float* dq_acc = static_cast<float*>(workspace);
    float* dvec = dq_acc + (size_t)rows * D;
    auto u16 = [](const void* p) { return static_cast<const uint16_t*>(p); };

    hipLaunchKernelGGL((fa_bwd_preprocess_kernel<Tag>), dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, stream,
                       u16(o), u16(dout), dvec, dq_acc, rows);

    int n_kblocks = (N + 127) / 128;
    long total = (long)B * H * n_kblocks;
    if (total > 0x7fffffffL) return FA_ERR_SHAPE;
    if (causal)
        hipLaunchKernelGGL((fa_bwd_kernel<Tag, true>), dim3((unsigned)total), dim3(256), 0, stream, u16(q), u16(k),
                           u16(v), u16(dout), lse, dvec, dq_acc, static_cast<uint16_t*>(dk),
                           static_cast<uint16_t*>(dv), N, n_kblocks, (int)total, scale);
    else
        hipLaunchKernelGGL((fa_bwd_kernel<Tag, false>), dim3((unsigned)total), dim3(256), 0, stream, u16(q), u16(k),
                           u16(v), u16(dout), lse, dvec, dq_acc, static_cast<uint16_t*>(dk),
                           static_cast<uint16_t*>(dv), N, n_kblocks, (int)total, scale);

    long n8 = rows * D / 8;
    hipLaunchKernelGGL((fa_bwd_convert_dq_kernel<Tag>), dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream,
                       dq_acc, static_cast<uint16_t*>(dq), n8, scale);
    return hipGetLastError() == hipSuccess ? FA_OK : FA_ERR_LAUNCH;
}

int launch_bwd(const void* q, const void* k, const void* v, const void* o, const float* lse, const void* dout,
               void* dq, void* dk, void* dv, void* workspace, int B, int H, int N, int d, float scale, int causal,
               int dtype, hipStream_t stream) {
    if (d != kBwdD) return FA_ERR_UNSUPPORTED;
    if (dtype == FA_BF16)
        return launch_bwd_t<bf16_tag>(q, k, v, o, lse, dout, dq, dk, dv, workspace, B, H, N, scale, causal, stream);
    if (dtype == FA_F16)
        return launch_bwd_t<f16_tag>(q, k, v, o, lse, dout, dq, dk, dv, workspace, B, H, N, scale, causal, stream);
    return FA_ERR_UNSUPPORTED;
}

}  // namespace fa
