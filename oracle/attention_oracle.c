/*
 * fp64 CPU oracle for exact scaled-dot-product attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the checker that the HIP kernels are
 * compared against; nothing on the product path may call it.  It shares no code
 * with the GPU library.
 *
 * What it computes is the plain definition (paper section 2.1):
 *     S = alpha * Q K^T,  P = softmax_rows(S),  O = P V,
 * with the row maximum subtracted before exponentiating, and, as the forward
 * algorithm's last step prescribes (Algorithm 1, epilogue), the row-wise
 * logsumexp  L_i = m_i + log(l_i)  (natural log of the alpha-scaled scores).
 * The backward pass is the chain rule of section 2.1:
 *     dV = P^T dO, dP = dO V^T, dS = dsoftmax(dP), dQ = alpha dS K, dK = alpha dS^T Q,
 * with dsoftmax written in the row form used by Algorithm 3:
 *     D_i = sum_k dO_ik O_ik,   dS_ij = P_ij (dP_ij - D_i).
 * No tiling, no online softmax, no fusion: one query row at a time.
 *
 * Causal mask (the paper only says "about half the entries"): key j is visible
 * to query i iff j <= i (square problem, diagonal included).
 *
 * Layout: all tensors are contiguous [B, H, N, d] doubles, d fastest;
 * L and D are [B, H, N].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One query row of one head.  Q row: q[d]; K, V: [N, d].  p is scratch of N doubles;
 * on return p[j] holds the normalised probability P_ij (0 for masked keys). */
static void attention_row(const double *q, const double *K, const double *V, int N, int d,
                          double alpha, int causal, int i, double *o, double *lse, double *p) {
    int nvis = causal ? (i + 1) : N; /* keys 0 .. nvis-1 are visible */
    double m = -INFINITY;
    for (int j = 0; j < nvis; ++j) {
        double s = 0.0;
        for (int k = 0; k < d; ++k) s += q[k] * K[(size_t)j * d + k];
        s *= alpha;
        p[j] = s;
        if (s > m) m = s;
    }
    double l = 0.0;
    for (int j = 0; j < nvis; ++j) {
        p[j] = exp(p[j] - m);
        l += p[j];
    }
    for (int k = 0; k < d; ++k) o[k] = 0.0;
    for (int j = 0; j < nvis; ++j) {
        p[j] /= l;
        for (int k = 0; k < d; ++k) o[k] += p[j] * V[(size_t)j * d + k];
    }
    for (int j = nvis; j < N; ++j) p[j] = 0.0;
    *lse = m + log(l);
}

/* Forward over the whole tensor (section 2.1; L from Algorithm 1's epilogue). */
void oracle_attn_fwd(const double *q, const double *k, const double *v, double *o, double *lse,
                     int B, int H, int N, int d, double alpha, int causal) {
    long total = (long)B * H * N;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 16)
        for (long r = 0; r < total; ++r) {
            long bh = r / N;
            int i = (int)(r % N);
            const double *Kh = k + (size_t)bh * N * d;
            const double *Vh = v + (size_t)bh * N * d;
            attention_row(q + (size_t)r * d, Kh, Vh, N, d, alpha, causal, i, o + (size_t)r * d,
                          lse + r, p);
        }
        free(p);
    }
}

/* Forward for a list of rows only.  rows[t] is a flat index into [B*H*N]; outputs are
 * packed: o_rows[t, :], lse_rows[t].  Rows are independent in the definition, so this is
 * the same computation restricted to the sampled rows. */
void oracle_attn_fwd_rows(const double *q, const double *k, const double *v, const int64_t *rows,
                          long nrows, double *o_rows, double *lse_rows, int B, int H, int N, int d,
                          double alpha, int causal) {
    (void)B;
    (void)H;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 4)
        for (long t = 0; t < nrows; ++t) {
            long r = rows[t];
            long bh = r / N;
            int i = (int)(r % N);
            attention_row(q + (size_t)r * d, k + (size_t)bh * N * d, v + (size_t)bh * N * d, N, d,
                          alpha, causal, i, o_rows + (size_t)t * d, lse_rows + t, p);
        }
        free(p);
    }
}

/* Backward over the whole tensor (section 2.1 chain rule, Algorithm 3's D and dS).
 * Recomputes P in fp64 from q, k, v; also returns the forward o, lse and D it used. */
void oracle_attn_bwd(const double *q, const double *k, const double *v, const double *dout,
                     double *o, double *lse, double *dvec, double *dq, double *dk, double *dv, int B,
                     int H, int N, int d, double alpha, int causal) {
    size_t hsz = (size_t)N * d;
    for (long bh = 0; bh < (long)B * H; ++bh) {
        const double *Qh = q + bh * hsz, *Kh = k + bh * hsz, *Vh = v + bh * hsz;
        const double *dOh = dout + bh * hsz;
        double *Oh = o + bh * hsz, *dQh = dq + bh * hsz, *dKh = dk + bh * hsz, *dVh = dv + bh * hsz;
        double *Lh = lse + (size_t)bh * N, *Dh = dvec + (size_t)bh * N;
        memset(dKh, 0, sizeof(double) * hsz);
        memset(dVh, 0, sizeof(double) * hsz);
#pragma omp parallel
        {
            double *p = (double *)malloc(sizeof(double) * (size_t)N);
            double *dKt = (double *)calloc(hsz, sizeof(double)); /* this thread's share of dK */
            double *dVt = (double *)calloc(hsz, sizeof(double));
#pragma omp for schedule(dynamic, 8)
            for (int i = 0; i < N; ++i) {
                const double *qi = Qh + (size_t)i * d;
                const double *doi = dOh + (size_t)i * d;
                double *oi = Oh + (size_t)i * d;
                double *dqi = dQh + (size_t)i * d;
                attention_row(qi, Kh, Vh, N, d, alpha, causal, i, oi, Lh + i, p);
                double D = 0.0;
                for (int c = 0; c < d; ++c) D += doi[c] * oi[c];
                Dh[i] = D;
                for (int c = 0; c < d; ++c) dqi[c] = 0.0;
                int nvis = causal ? (i + 1) : N;
                for (int j = 0; j < nvis; ++j) {
                    const double *kj = Kh + (size_t)j * d, *vj = Vh + (size_t)j * d;
                    double dp = 0.0;
                    for (int c = 0; c < d; ++c) dp += doi[c] * vj[c]; /* dP_ij = dO_i . V_j */
                    double ds = p[j] * (dp - D);                      /* dS_ij */
                    for (int c = 0; c < d; ++c) {
                        dqi[c] += alpha * ds * kj[c];                 /* dQ = alpha dS K   */
                        dKt[(size_t)j * d + c] += alpha * ds * qi[c]; /* dK = alpha dS^T Q */
                        dVt[(size_t)j * d + c] += p[j] * doi[c];      /* dV = P^T dO       */
                    }
                }
            }
#pragma omp critical
            {
                for (size_t t = 0; t < hsz; ++t) {
                    dKh[t] += dKt[t];
                    dVh[t] += dVt[t];
                }
            }
            free(p);
            free(dKt);
            free(dVt);
        }
    }
}

/* dQ of sampled query rows only (same arithmetic as oracle_attn_bwd, one row at a time):
 * rows[t] is a flat index into B*H*N; dq_rows is [n_rows, d].  Cost O(n_rows N d). */
void oracle_attn_bwd_dq_rows(const double *q, const double *k, const double *v, const double *dout,
                             const int64_t *rows, long n_rows, double *dq_rows, int B, int H, int N, int d,
                             double alpha, int causal) {
    (void)B;
    (void)H;
    size_t hsz = (size_t)N * d;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)N);
        double *oi = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 1)
        for (long t = 0; t < n_rows; ++t) {
            long bh = rows[t] / N;
            int i = (int)(rows[t] % N);
            const double *Kh = k + bh * hsz, *Vh = v + bh * hsz;
            const double *qi = q + bh * hsz + (size_t)i * d, *doi = dout + bh * hsz + (size_t)i * d;
            double *dqi = dq_rows + (size_t)t * d, lse;
            attention_row(qi, Kh, Vh, N, d, alpha, causal, i, oi, &lse, p);
            double D = 0.0;
            for (int c = 0; c < d; ++c) D += doi[c] * oi[c];
            for (int c = 0; c < d; ++c) dqi[c] = 0.0;
            int nvis = causal ? (i + 1) : N;
            for (int j = 0; j < nvis; ++j) {
                const double *kj = Kh + (size_t)j * d, *vj = Vh + (size_t)j * d;
                double dp = 0.0;
                for (int c = 0; c < d; ++c) dp += doi[c] * vj[c];
                double ds = p[j] * (dp - D);
                for (int c = 0; c < d; ++c) dqi[c] += alpha * ds * kj[c];
            }
        }
        free(p);
        free(oi);
    }
}

/* dK and dV of the key rows [j0, j1) of ONE head (q, k, v, dout: [N, d]; dk, dv: [j1-j0, d]).
 * Every query that sees one of these keys contributes: all N of them without a mask, the
 * queries i >= j0 under the causal mask -- so for keys near the end of a long causal problem
 * this costs O((N - j0) N d) instead of O(N^2 d). */
void oracle_attn_bwd_dkdv_keys(const double *q, const double *k, const double *v, const double *dout, int j0,
                               int j1, double *dk, double *dv, int N, int d, double alpha, int causal) {
    size_t outsz = (size_t)(j1 - j0) * d;
    memset(dk, 0, sizeof(double) * outsz);
    memset(dv, 0, sizeof(double) * outsz);
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)N);
        double *oi = (double *)malloc(sizeof(double) * (size_t)d);
        double *dkt = (double *)calloc(outsz + 1, sizeof(double)); /* this thread's share */
        double *dvt = (double *)calloc(outsz + 1, sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int i = causal ? j0 : 0; i < N; ++i) {
            const double *qi = q + (size_t)i * d, *doi = dout + (size_t)i * d;
            double lse;
            attention_row(qi, k, v, N, d, alpha, causal, i, oi, &lse, p);
            double D = 0.0;
            for (int c = 0; c < d; ++c) D += doi[c] * oi[c];
            int nvis = causal ? (i + 1) : N;
            for (int j = j0; j < j1 && j < nvis; ++j) {
                const double *vj = v + (size_t)j * d;
                double dp = 0.0;
                for (int c = 0; c < d; ++c) dp += doi[c] * vj[c];
                double ds = p[j] * (dp - D);
                for (int c = 0; c < d; ++c) {
                    dkt[(size_t)(j - j0) * d + c] += alpha * ds * qi[c];
                    dvt[(size_t)(j - j0) * d + c] += p[j] * doi[c];
                }
            }
        }
#pragma omp critical
        {
            for (size_t t = 0; t < outsz; ++t) {
                dk[t] += dkt[t];
                dv[t] += dvt[t];
            }
        }
        free(p);
        free(oi);
        free(dkt);
        free(dvt);
    }
}

/* The probability matrix of one head, P[N, N] (for invariants such as rows summing to 1). */
void oracle_attn_probs(const double *q, const double *k, const double *v, double *P, int N, int d,
                       double alpha, int causal) {
    double *o = (double *)malloc(sizeof(double) * (size_t)d);
    double lse;
    for (int i = 0; i < N; ++i)
        attention_row(q + (size_t)i * d, k, v, N, d, alpha, causal, i, o, &lse, P + (size_t)i * N);
    free(o);
}
