/*
 * CPU ORACLE -- test infrastructure, not the product.
 *
 * Plain element loops for the three per-element operations of Slow Momentum
 * (Algorithm 1) with the base-optimizer directions of Table C.1 (Appendix C).
 * Nothing here is blocked, fused or reordered beyond what those passages
 * state.  The file is compiled twice from the same source:
 *
 *   -DREAL=double  every state value and every operation in fp64 (the
 *                  reference the GPU path is checked against);
 *   -DREAL=float   every state value in fp32, one rounding per operation
 *                  (build with -ffp-contract=off): the fp32 noise floor.
 *
 * Gradients arrive as fp32 values (a bf16 gradient has already been widened,
 * which is exact) and are converted to REAL on use.  Only tests, the smoke
 * check and the benchmark's CPU-baseline leg may call this code; it shares
 * nothing with the HIP path.
 *
 * Every element index j evolves independently of all others (all operations
 * below are element-wise; the only coupling is across the m workers at one
 * j), so the loop over j carries an OpenMP "parallel for": it changes no
 * element's arithmetic or its order.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (closed forms, special-case reductions of Section 2, library optimizers).
 */
#include <math.h>
#include <stdint.h>

#ifndef REAL
#define REAL double
#endif

#if defined(ORACLE_F32)
#define R_SQRT sqrtf
#define R_POW powf
#else
#define R_SQRT sqrt
#define R_POW pow
#endif

/* Size in bytes of REAL, so the caller can check which build it loaded. */
int oracle_real_bytes(void) { return (int)sizeof(REAL); }

/* Threads the "parallel for" loops below run on (for the timing report). */
#ifdef _OPENMP
#include <omp.h>
int oracle_num_threads(void) { return omp_get_max_threads(); }
#else
int oracle_num_threads(void) { return 1; }
#endif

/*
 * One base-optimizer step of one worker, SGD with Nesterov momentum
 * (Table C.1, row "SGD"; Algorithm 1 line 4):
 *     h_{k+1} = mu * h_k + grad
 *     d_k     = mu * h_{k+1} + grad
 *     x_{k+1} = x_k - lr * d_k
 * Weight decay (Appendix A.2/A.3 name only the factor 1e-4) is read as the
 * coupled L2 term: grad = g + wd * x_k, with x_k the value before the step,
 * and that sum feeds both h and d.
 */
void oracle_sgd_nesterov_step(REAL *x, REAL *h, const float *g, int64_t d,
                              double lr_, double mu_, double wd_)
{
    const REAL lr = (REAL)lr_, mu = (REAL)mu_, wd = (REAL)wd_;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        REAL grad = (REAL)g[j] + wd * x[j];
        REAL hn = mu * h[j] + grad;
        REAL dir = mu * hn + grad;
        h[j] = hn;
        x[j] = x[j] - lr * dir;
    }
}

/*
 * One base-optimizer step of one worker, Adam (Table C.1, row "Adam"):
 *     h_{k+1} = b1 * h_k + (1 - b1) * grad
 *     v_{k+1} = b2 * v_k + (1 - b2) * grad^2        (element-wise square)
 *     hhat = h_{k+1} / (1 - b1^l),  vhat = v_{k+1} / (1 - b2^l)
 *     d_k  = hhat / (sqrt(vhat) + eps)              (eps after the root)
 *     x_{k+1} = x_k - lr * d_k
 * l is the number of moment updates applied so far INCLUDING this one (the
 * table's printed exponent starts at 0, which would divide by zero on the
 * first step; the caller passes l = 1, 2, ...).  Weight decay, if non-zero,
 * is the same coupled term as for SGD.
 */
void oracle_adam_step(REAL *x, REAL *h, REAL *v, const float *g, int64_t d,
                      double lr_, double b1_, double b2_, double eps_,
                      double wd_, int64_t l)
{
    const REAL lr = (REAL)lr_, b1 = (REAL)b1_, b2 = (REAL)b2_;
    const REAL eps = (REAL)eps_, wd = (REAL)wd_;
    const REAL one = (REAL)1;
    const REAL c1 = one - R_POW(b1, (REAL)l);
    const REAL c2 = one - R_POW(b2, (REAL)l);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        REAL grad = (REAL)g[j] + wd * x[j];
        REAL gsq = grad * grad;
        REAL hn = b1 * h[j] + (one - b1) * grad;
        REAL vn = b2 * v[j] + (one - b2) * gsq;
        REAL hhat = hn / c1;
        REAL vhat = vn / c2;
        REAL dir = hhat / (R_SQRT(vhat) + eps);
        h[j] = hn;
        v[j] = vn;
        x[j] = x[j] - lr * dir;
    }
}

/*
 * The outer step (Algorithm 1 lines 6-8, Eq. (2) and (3)), then the copy of
 * the new outer iterate into every worker's replica (Section 2: the iterates
 * are identical on all workers after the exact average).
 *   xw : m replicas, worker-major, replica i at xw + i*d
 *   line 6:  xbar = (1/m) * sum_{i=0}^{m-1} x^{(i)}   summed in this order
 *   line 7:  u  <- beta * u + (x0 - xbar) / lr
 *   line 8:  x0 <- x0 - alpha * lr * u
 */
void oracle_outer_step(REAL *xw, int m, int64_t d, REAL *x0, REAL *u,
                       double lr_, double alpha_, double beta_)
{
    const REAL lr = (REAL)lr_, alpha = (REAL)alpha_, beta = (REAL)beta_;
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        REAL s = xw[j];
        for (int i = 1; i < m; ++i)
            s = s + xw[(int64_t)i * d + j];
        REAL xbar = s / (REAL)m;
        REAL diff = x0[j] - xbar;
        REAL un = beta * u[j] + diff / lr;
        REAL xn = x0[j] - (alpha * lr) * un;
        u[j] = un;
        x0[j] = xn;
        for (int i = 0; i < m; ++i)
            xw[(int64_t)i * d + j] = xn;
    }
}

/*
 * Buffer strategy "average" (Appendix B.4, strategy 3; for the momentum
 * buffer also Algorithm C.4, "double averaging"): every worker's buffer is
 * replaced by the mean of the m workers' buffers, summed in worker order.
 *   bw : m buffers, worker-major, buffer i at bw + i*d
 */
void oracle_average_buffers(REAL *bw, int m, int64_t d)
{
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < d; ++j) {
        REAL s = bw[j];
        for (int i = 1; i < m; ++i)
            s = s + bw[(int64_t)i * d + j];
        REAL mean = s / (REAL)m;
        for (int i = 0; i < m; ++i)
            bw[(int64_t)i * d + j] = mean;
    }
}

/*
 * One mixing step of stochastic gradient push among the m workers
 * (Algorithm C.1: send / receive / "update model parameters" / "update
 * de-biased factors"; matrix form X_{k+1} = X_{k+1/2} P^T of Appendix C.1).
 * Every worker i has at most one in-neighbour in_peer[i] besides itself
 * (in_peer[i] == i: none), and a sender splits its mass uniformly over itself
 * and its receivers, which makes P column-stochastic:
 *     p(i,j) = 1 / (1 + outdeg(j))  for j == i or j == in_peer[i],  else 0.
 *   xw : m replicas (worker-major), mixed in place
 *   w  : the m push-sum weights, mixed with the same P
 */
void oracle_mix_step(REAL *xw, REAL *w, int m, int64_t d, const int32_t *in_peer)
{
    REAL share[m];                      /* 1 / (1 + outdeg(j)) */
    for (int j = 0; j < m; ++j) {
        int outdeg = 0;
        for (int i = 0; i < m; ++i)
            if (i != j && in_peer[i] == j) ++outdeg;
        share[j] = (REAL)1 / (REAL)(1 + outdeg);
    }
    REAL wold[m];
    for (int i = 0; i < m; ++i) wold[i] = w[i];
    for (int i = 0; i < m; ++i) {
        int j = in_peer[i];
        w[i] = share[i] * wold[i];
        if (j != i) w[i] = w[i] + share[j] * wold[j];
    }
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < d; ++e) {
        REAL old[m];
        for (int i = 0; i < m; ++i) old[i] = xw[(int64_t)i * d + e];
        for (int i = 0; i < m; ++i) {
            int j = in_peer[i];
            REAL v = share[i] * old[i];
            if (j != i) v = v + share[j] * old[j];
            xw[(int64_t)i * d + e] = v;
        }
    }
}
