/*
 * The C ABI used from plain C (no Python, no C++): a Slow Momentum run with
 * plain SGD as base optimizer and CONSTANT per-worker gradients c_i, checked
 * against the closed form that Eq. (2)-(3) of the paper give for that case:
 *     u_t      = tau * cbar * (1 - beta^t) / (1 - beta)
 *     x_{T,0}  = x_{0,0} - alpha * gamma * tau * cbar * sum_{t=1..T} (1 - beta^t)/(1 - beta)
 * (cbar = mean of the c_i), followed by one push-sum mixing step on the consensus point
 * (Algorithm C.1) whose de-biased parameters must give that point back.
 * Prints "OK" and returns 0 on success.
 * Built by __graft_entry__.build() into tests/abi_c_check; run by the GPU tests.
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../include/slowmo.h"

#define HIPCHECK(call)                                                        \
    do {                                                                      \
        hipError_t e_ = (call);                                               \
        if (e_ != hipSuccess) {                                               \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            return 2;                                                         \
        }                                                                     \
    } while (0)
#define SMCHECK(call, ctx)                                                    \
    do {                                                                      \
        slowmo_status s_ = (call);                                            \
        if (s_ != SLOWMO_OK) {                                                \
            printf("slowmo error %d (%s) at line %d\n", (int)s_, slowmo_last_error(ctx), __LINE__); \
            return 3;                                                         \
        }                                                                     \
    } while (0)

enum { M = 3, NT = 2, TAU = 4, ROUNDS = 5 };

int main(void) {
    const int64_t numel[NT] = {1000, 37};
    const float lr = 0.05f, alpha = 0.75f, beta = 0.5f;
    slowmo_config cfg = {0};
    cfg.m = M;
    cfg.tau = TAU;
    cfg.alpha = alpha;
    cfg.beta = beta;
    cfg.base = SLOWMO_SGD_NESTEROV;       /* momentum 0, wd 0: plain SGD */
    cfg.policy = SLOWMO_BUF_RESET;
    cfg.grad_dtype = SLOWMO_F32;

    float *params[M * NT];
    const void *grads[M * NT];
    float *host = malloc(sizeof(float) * 1000);
    for (int i = 0; i < M; ++i) {
        for (int j = 0; j < NT; ++j) {
            float *p, *g;
            HIPCHECK(hipMalloc((void **)&p, sizeof(float) * (size_t)numel[j]));
            HIPCHECK(hipMalloc((void **)&g, sizeof(float) * (size_t)numel[j]));
            for (int64_t e = 0; e < numel[j]; ++e) host[e] = 1.0f + 0.001f * (float)e;      /* x_{0,0} */
            HIPCHECK(hipMemcpy(p, host, sizeof(float) * (size_t)numel[j], hipMemcpyHostToDevice));
            for (int64_t e = 0; e < numel[j]; ++e) host[e] = (float)(i + 1) * 0.25f;        /* c_i */
            HIPCHECK(hipMemcpy(g, host, sizeof(float) * (size_t)numel[j], hipMemcpyHostToDevice));
            params[i * NT + j] = p;
            grads[i * NT + j] = g;
        }
    }
    size_t bytes = slowmo_state_bytes(&cfg, NT, numel);
    if (!bytes) { printf("slowmo_state_bytes failed: %s\n", slowmo_last_error(NULL)); return 3; }
    void *state;
    HIPCHECK(hipMalloc(&state, bytes));
    slowmo_ctx *ctx = NULL;
    SMCHECK(slowmo_create(&ctx, &cfg, NT, numel, params, state, bytes, NULL), NULL);
    if (slowmo_outer_step(ctx, lr, NULL) != SLOWMO_ERR_STATE) { printf("missing STATE error\n"); return 4; }
    for (int t = 0; t < ROUNDS; ++t) {
        for (int k = 0; k < TAU - 1; ++k) SMCHECK(slowmo_local_step(ctx, grads, lr, NULL), ctx);
        if (t % 2) {
            SMCHECK(slowmo_local_outer_step(ctx, grads, lr, lr, NULL), ctx);
        } else {
            SMCHECK(slowmo_local_step(ctx, grads, lr, NULL), ctx);
            SMCHECK(slowmo_outer_step(ctx, lr, NULL), ctx);
        }
    }
    HIPCHECK(hipDeviceSynchronize());
    int64_t t_done = 0;
    SMCHECK(slowmo_get_counters(ctx, &t_done, NULL, NULL), ctx);
    if (t_done != ROUNDS) { printf("counter t = %lld\n", (long long)t_done); return 4; }

    const double cbar = 0.25 * (1 + 2 + 3) / 3.0;
    double geo_sum = 0, geo_last = 0;
    for (int t = 1; t <= ROUNDS; ++t) { geo_last = (1 - pow(beta, t)) / (1 - beta); geo_sum += geo_last; }
    double worst = 0;
    for (int j = 0; j < NT; ++j) {
        float *du;
        SMCHECK(slowmo_get_buffer(ctx, SLOWMO_BUF_U, 0, j, &du), ctx);
        for (int i = 0; i < M; ++i) {
            HIPCHECK(hipMemcpy(host, params[i * NT + j], sizeof(float) * (size_t)numel[j], hipMemcpyDeviceToHost));
            for (int64_t e = 0; e < numel[j]; ++e) {
                double want = (1.0 + 0.001 * (double)e) - (double)alpha * lr * TAU * cbar * geo_sum;
                double err = fabs(host[e] - want) / (1 + fabs(want));
                if (err > worst) worst = err;
            }
        }
        HIPCHECK(hipMemcpy(host, du, sizeof(float) * (size_t)numel[j], hipMemcpyDeviceToHost));
        for (int64_t e = 0; e < numel[j]; ++e) {
            double err = lr * fabs(host[e] - TAU * cbar * geo_last) / (1 + lr * TAU * cbar * geo_last);
            if (err > worst) worst = err;
        }
    }
    /* Push-sum (Algorithm C.1) on the consensus point: worker 0 sends to everybody.  Its mass is
     * split over M workers, so x^(0) = x/M, x^(i) = x + x/M, w = (1/M, 1 + 1/M, ...), and the
     * de-biased parameters z^(i) = x^(i) / w_i are the consensus point again on every worker. */
    {
        const int32_t star[M] = {0};
        float w[M], *z[M * NT];
        SMCHECK(slowmo_mix_step(ctx, star, NULL), ctx);
        SMCHECK(slowmo_get_pushsum_weights(ctx, w), ctx);
        for (int i = 0; i < M; ++i) {
            double want_w = i == 0 ? 1.0 / M : 1.0 + 1.0 / M;
            if (fabs(w[i] - want_w) > 1e-6) { printf("push-sum weight %d is %g\n", i, w[i]); return 6; }
            for (int j = 0; j < NT; ++j)
                HIPCHECK(hipMalloc((void **)&z[i * NT + j], sizeof(float) * (size_t)numel[j]));
        }
        SMCHECK(slowmo_debias(ctx, z, NULL), ctx);
        HIPCHECK(hipDeviceSynchronize());
        for (int i = 0; i < M; ++i) {
            for (int j = 0; j < NT; ++j) {
                float *biased = malloc(sizeof(float) * (size_t)numel[j]);
                HIPCHECK(hipMemcpy(host, z[i * NT + j], sizeof(float) * (size_t)numel[j], hipMemcpyDeviceToHost));
                HIPCHECK(hipMemcpy(biased, params[i * NT + j], sizeof(float) * (size_t)numel[j], hipMemcpyDeviceToHost));
                for (int64_t e = 0; e < numel[j]; ++e) {
                    double want = (1.0 + 0.001 * (double)e) - (double)alpha * lr * TAU * cbar * geo_sum;
                    double err = fabs(host[e] - want) / (1 + fabs(want));
                    if (err > worst) worst = err;
                    err = fabs(biased[e] - want * (i == 0 ? 1.0 / M : 1.0 + 1.0 / M)) / (1 + fabs(want));
                    if (err > worst) worst = err;
                }
                free(biased);
                HIPCHECK(hipFree(z[i * NT + j]));
            }
        }
    }
    SMCHECK(slowmo_destroy(ctx), NULL);
    if (worst > 1e-5) { printf("closed form missed: worst error %.3e\n", worst); return 5; }
    printf("OK worst error %.3e\n", worst);
    return 0;
}
