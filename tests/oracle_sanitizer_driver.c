/* Runs the CPU oracle's element loops under AddressSanitizer / UBSan (host
 * only): odd sizes, m = 1, an empty range, every entry point.  Prints "OK".
 * Built by tests/test_oracle_sanitized.py together with oracle/slowmo_oracle.c. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#ifndef REAL
#define REAL double
#endif

void oracle_sgd_nesterov_step(REAL *x, REAL *h, const float *g, int64_t d, double lr, double mu, double wd);
void oracle_adam_step(REAL *x, REAL *h, REAL *v, const float *g, int64_t d, double lr, double b1,
                      double b2, double eps, double wd, int64_t l);
void oracle_outer_step(REAL *xw, int m, int64_t d, REAL *x0, REAL *u, double lr, double alpha, double beta);
void oracle_average_buffers(REAL *bw, int m, int64_t d);
void oracle_mix_step(REAL *xw, REAL *w, int m, int64_t d, const int32_t *in_peer);

static REAL *reals(int64_t n, REAL v) {
    REAL *p = malloc(sizeof(REAL) * (size_t)(n > 0 ? n : 1));
    for (int64_t i = 0; i < n; ++i) p[i] = v + (REAL)i * (REAL)0.01;
    return p;
}

int main(void) {
    const int ms[] = {1, 3, 5};
    const int64_t ds[] = {0, 1, 7, 1025};
    for (unsigned a = 0; a < sizeof ms / sizeof ms[0]; ++a) {
        for (unsigned b = 0; b < sizeof ds / sizeof ds[0]; ++b) {
            const int m = ms[a];
            const int64_t d = ds[b];
            REAL *x = reals(m * d, 1), *h = reals(m * d, 0), *v = reals(m * d, 0.5);
            REAL *x0 = reals(d, 1), *u = reals(d, 0), *w = reals(m, 1);
            float *g = malloc(sizeof(float) * (size_t)(m * d > 0 ? m * d : 1));
            int32_t *peer = malloc(sizeof(int32_t) * (size_t)m);
            for (int64_t i = 0; i < m * d; ++i) g[i] = (float)(i % 13) - 6.0f;
            for (int i = 0; i < m; ++i) { peer[i] = (i + 1) % m; w[i] = 1; }
            for (int step = 1; step <= 3; ++step) {
                for (int i = 0; i < m; ++i) {
                    oracle_sgd_nesterov_step(x + i * d, h + i * d, g + i * d, d, 0.1, 0.9, 1e-4);
                    oracle_adam_step(x + i * d, h + i * d, v + i * d, g + i * d, d, 1e-3, 0.9, 0.98, 1e-8, 0.0, step);
                }
                oracle_mix_step(x, w, m, d, peer);
            }
            oracle_average_buffers(h, m, d);
            oracle_outer_step(x, m, d, x0, u, 0.1, 1.0, 0.6);
            for (int64_t j = 0; j < d; ++j)
                if (x[j] != x0[j] || x[(m - 1) * d + j] != x0[j]) { printf("consensus broken\n"); return 1; }
            free(x); free(h); free(v); free(x0); free(u); free(w); free(g); free(peer);
        }
    }
    printf("OK\n");
    return 0;
}
