/* Runs every entry point of oracle/attention_oracle.c on small ragged problems; built with
 * -fsanitize=address,undefined by tests/test_sanitizers_host.py, which only checks that it exits 0
 * (any out-of-bounds access or undefined operation aborts it). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void oracle_attn_fwd(const double*, const double*, const double*, double*, double*, int, int, int, int, double, int);
void oracle_attn_fwd_rows(const double*, const double*, const double*, const int64_t*, long, double*, double*, int, int,
                          int, int, double, int);
void oracle_attn_bwd(const double*, const double*, const double*, const double*, double*, double*, double*, double*,
                     double*, double*, int, int, int, int, double, int);
void oracle_attn_bwd_dq_rows(const double*, const double*, const double*, const double*, const int64_t*, long, double*,
                             int, int, int, int, double, int);
void oracle_attn_bwd_dkdv_keys(const double*, const double*, const double*, const double*, int, int, double*, double*,
                               int, int, double, int);
void oracle_attn_probs(const double*, const double*, const double*, double*, int, int, double, int);

static double* filled(size_t n, unsigned seed) {
    double* p = malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) {
        seed = seed * 1664525u + 1013904223u;
        p[i] = ((double)(seed >> 8) / (1 << 24)) * 2.0 - 1.0;
    }
    return p;
}

int main(void) {
    const int shapes[][4] = {{1, 1, 1, 1}, {2, 3, 7, 5}, {1, 2, 33, 8}};
    for (unsigned s = 0; s < sizeof(shapes) / sizeof(shapes[0]); ++s) {
        const int B = shapes[s][0], H = shapes[s][1], N = shapes[s][2], d = shapes[s][3];
        const size_t n = (size_t)B * H * N * d, rows = (size_t)B * H * N;
        double *q = filled(n, 1), *k = filled(n, 2), *v = filled(n, 3), *dout = filled(n, 4);
        double *o = malloc(n * 8), *dq = malloc(n * 8), *dk = malloc(n * 8), *dv = malloc(n * 8);
        double *lse = malloc(rows * 8), *D = malloc(rows * 8), *P = malloc((size_t)N * N * 8);
        int64_t pick[3] = {0, (int64_t)rows / 2, (int64_t)rows - 1};
        double *orow = malloc(3 * d * 8), *lrow = malloc(3 * 8);
        for (int causal = 0; causal < 2; ++causal) {
            oracle_attn_fwd(q, k, v, o, lse, B, H, N, d, 0.3, causal);
            oracle_attn_fwd_rows(q, k, v, pick, 3, orow, lrow, B, H, N, d, 0.3, causal);
            oracle_attn_bwd(q, k, v, dout, o, lse, D, dq, dk, dv, B, H, N, d, 0.3, causal);
            oracle_attn_bwd_dq_rows(q, k, v, dout, pick, 3, orow, B, H, N, d, 0.3, causal);
            oracle_attn_bwd_dkdv_keys(q, k, v, dout, N / 2, N, dk, dv, N, d, 0.3, causal);
            oracle_attn_probs(q, k, v, P, N, d, 0.3, causal);
        }
        free(q); free(k); free(v); free(dout); free(o); free(dq); free(dk); free(dv);
        free(lse); free(D); free(P); free(orow); free(lrow);
    }
    puts("oracle sanitizer run: ok");
    return 0;
}
