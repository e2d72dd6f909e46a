/*
 * CPU oracle for the multi-LoRA linear layer (TEST INFRASTRUCTURE, not product code).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code with the HIP library and is never a fallback for it.
 *
 * What it computes is the plain definition of the layer, one adapter segment at a
 * time, in fp64, with naive triple loops: every output element is one plain sum over
 * the contraction index in increasing order; only the outermost loop is
 * OpenMP-parallel; there is no blocking, no fusion and no reordering of a sum:
 *
 *   LoRA residual branch  Y = XW + XAB                      (paper Sec. 2.1)
 *   S = XA, L = SB, Y = S_i B_i + Y_base                    (paper Sec. 5.1)
 *   dS = scale * dY B_i^T, dX = dS A_i^T,
 *   dA_i = X_i^T dS_i, dB_i = S_i^T dY_i                    (paper Sec. 5.1, backward)
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - the LoRA term carries the per-adapter scale s_i:  Y_i = X_i W + s_i (X_i A_i) B_i;
 *     the cached S_i = X_i A_i is unscaled, so dB_i = s_i S_i^T dY_i (the paper's
 *     dB formula drops the scale; finite differences in the tests settle it);
 *   - dX includes the frozen-weight term: dX_i = dY_i W^T + dS_i A_i^T;
 *   - W is [k,n], A_i is [k,r_i], B_i is [r_i,n], all row-major (paper's orientation).
 *
 * Inputs are float32 arrays holding exactly the values the GPU receives (a bf16
 * value widens to float32 without rounding); everything is widened to double before
 * any arithmetic and every sum is accumulated in double.  Outputs are double.
 *
 * Row / column index lists let a caller ask for a sample of the outputs of a big
 * problem; each requested element is still the full, unsampled contraction.
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int mlo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void mlo_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* S[t,rho] = sum_kappa X[t,kappa] * A[kappa,rho]      (Sec. 5.1: S = XA)
 * X: Ti rows with row stride ldx (>= k); A: [k,r]; S: [Ti,r] double. */
void mlo_shrink(int64_t Ti, int64_t k, int64_t r, const float* X, int64_t ldx,
                const float* A, double* S) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < Ti; ++t) {
        double* s = S + t * r;
        for (int64_t rho = 0; rho < r; ++rho) s[rho] = 0.0;
        for (int64_t kappa = 0; kappa < k; ++kappa) {
            const double x = (double)X[t * ldx + kappa];
            for (int64_t rho = 0; rho < r; ++rho) s[rho] += x * (double)A[kappa * r + rho];
        }
    }
}

/* Y[a,b] = sum_kappa X[ri[a],kappa] W[kappa,ci[b]] + s * sum_rho S[ri[a],rho] B[rho,ci[b]]
 * (Sec. 2.1 with the scale reading; Sec. 5.1: Y = S_i B_i + Y_base).
 * X: segment rows (row stride ldx), S: [Ti,r] double for the same segment,
 * ri: nr row indices local to the segment (NULL = 0..nr-1),
 * ci: nc column indices (NULL = 0..nc-1).  Y: [nr,nc] double.
 * The base term and the LoRA term are accumulated separately and added once. */
void mlo_fwd_y(int64_t nr, const int64_t* ri, int64_t nc, const int64_t* ci,
               int64_t k, int64_t n, int64_t r, double s,
               const float* X, int64_t ldx, const float* W,
               const double* S, const float* B, double* Y, double* Ybase_opt) {
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < nr; ++a) {
        const int64_t t = ri ? ri[a] : a;
        double* y = Y + a * nc;
        for (int64_t b = 0; b < nc; ++b) y[b] = 0.0;
        for (int64_t kappa = 0; kappa < k; ++kappa) {
            const double x = (double)X[t * ldx + kappa];
            const float* w = W + kappa * n;
            if (ci) for (int64_t b = 0; b < nc; ++b) y[b] += x * (double)w[ci[b]];
            else    for (int64_t b = 0; b < nc; ++b) y[b] += x * (double)w[b];
        }
        if (Ybase_opt) for (int64_t b = 0; b < nc; ++b) Ybase_opt[a * nc + b] = y[b];
        for (int64_t b = 0; b < nc; ++b) {
            const int64_t nu = ci ? ci[b] : b;
            double l = 0.0;
            for (int64_t rho = 0; rho < r; ++rho) l += S[t * r + rho] * (double)B[rho * n + nu];
            y[b] += s * l;
        }
    }
}

/* dS[t,rho] = s * sum_nu dY[t,nu] * B[rho,nu]      (Sec. 5.1: dS = scale dY B_i^T) */
void mlo_dshrink(int64_t Ti, int64_t n, int64_t r, double s, const float* dY, int64_t lddy,
                 const float* B, double* dS) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < Ti; ++t) {
        for (int64_t rho = 0; rho < r; ++rho) {
            double acc = 0.0;
            for (int64_t nu = 0; nu < n; ++nu) acc += (double)dY[t * lddy + nu] * (double)B[rho * n + nu];
            dS[t * r + rho] = s * acc;
        }
    }
}

/* dX[a,b] = sum_nu dY[ri[a],nu] W[ci[b],nu] + sum_rho dS[ri[a],rho] A[ci[b],rho]
 * (Sec. 5.1: dX = dS A_i^T, plus the frozen-weight input gradient dY W^T). */
void mlo_bwd_dx(int64_t nr, const int64_t* ri, int64_t nc, const int64_t* ci,
                int64_t k, int64_t n, int64_t r,
                const float* dY, int64_t lddy, const float* W,
                const double* dS, const float* A, double* dX) {
    (void)k;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < nr; ++a) {
        const int64_t t = ri ? ri[a] : a;
        for (int64_t b = 0; b < nc; ++b) {
            const int64_t kappa = ci ? ci[b] : b;
            double base = 0.0;
            for (int64_t nu = 0; nu < n; ++nu) base += (double)dY[t * lddy + nu] * (double)W[kappa * n + nu];
            double lora = 0.0;
            for (int64_t rho = 0; rho < r; ++rho) lora += dS[t * r + rho] * (double)A[kappa * r + rho];
            dX[a * nc + b] = base + lora;
        }
    }
}

/* dA[b,rho] = sum_{t in segment} X[t,ci[b]] * dS[t,rho]      (Sec. 5.1: dA_i = X_i^T dS_i)
 * ci: nc row indices of dA (NULL = all k rows, nc == k).  dA: [nc,r] double. */
void mlo_wgrad_a(int64_t Ti, int64_t k, int64_t r, int64_t nc, const int64_t* ci,
                 const float* X, int64_t ldx, const double* dS, double* dA) {
    (void)k;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nc; ++b) {
        const int64_t kappa = ci ? ci[b] : b;
        double* d = dA + b * r;
        for (int64_t rho = 0; rho < r; ++rho) d[rho] = 0.0;
        for (int64_t t = 0; t < Ti; ++t) {
            const double x = (double)X[t * ldx + kappa];
            for (int64_t rho = 0; rho < r; ++rho) d[rho] += x * dS[t * r + rho];
        }
    }
}

/* dB[rho,b] = s * sum_{t in segment} S[t,rho] * dY[t,ci[b]]   (Sec. 5.1: dB_i = S_i^T dY_i,
 * times s_i because S is cached unscaled).  ci: nc column indices (NULL = all n).
 * dB: [r,nc] double. */
void mlo_wgrad_b(int64_t Ti, int64_t n, int64_t r, double s, int64_t nc, const int64_t* ci,
                 const double* S, const float* dY, int64_t lddy, double* dB) {
    (void)n;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < nc; ++b) {
        const int64_t nu = ci ? ci[b] : b;
        for (int64_t rho = 0; rho < r; ++rho) dB[rho * nc + b] = 0.0;
        for (int64_t t = 0; t < Ti; ++t) {
            const double g = (double)dY[t * lddy + nu];
            for (int64_t rho = 0; rho < r; ++rho) dB[rho * nc + b] += S[t * r + rho] * g;
        }
        for (int64_t rho = 0; rho < r; ++rho) dB[rho * nc + b] *= s;
    }
}
