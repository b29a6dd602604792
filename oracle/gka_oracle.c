/*
 * gka_oracle.c -- plain fp64 CPU oracle for the Gated KalmaNet (GKA) layer forward pass.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is
 * deliberately slow and literal.  It shares no code, header, table or helper with the HIP
 * path and must never be linked into, imported by, or called from the product library.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What it computes (paper Section 4.1, Eq. (CH)), per (batch, head) pair and token t:
 *     H_t = gamma_t * H_{t-1} + k_t k_t^T          (d_k x d_k)
 *     U_t = gamma_t * U_{t-1} + v_t k_t^T          (d_v x d_k)
 *     xhat_t = CH(H_t + lambda_t I, q_t, r)        (Algorithm 1, r iterations)
 *     y_t = U_t xhat_t
 * with eigenvalue bounds L = ||H_t||_F + lambda_t and mu = lambda_t (Section 4.1,
 * "Adaptive Regularization").  H_t is formed explicitly for every token: no chunking,
 * no fusion, no reordering.  lambda_t is either given per token or, when the lambda
 * array is NULL, set by the paper's rule lambda_t = a * ||H_t||_F.
 *
 * Pins (tests/test_oracle_pins.py): printed kappa=51 constants of the Remark in
 * Appendix B.1; the omega-schedule lemmas of Appendix B.1; the Chebyshev-polynomial closed
 * form of Algorithm 1 on an eigen-decomposed matrix; the single-token closed form; the
 * direct Cholesky solve of the ridge problem Eq. (rls) / its closed form in Section 4.1 and
 * convergence towards it; the ungated constant-lambda Kalman/RLS recursion Eq. (KF); the
 * chunk identities of Section 4.2.1; sequence-split and decode hand-off; the write gate beta
 * (equivalence with sqrt(beta)-scaled k and v, single-token closed form); the alpha-connection
 * (single-token closed form, interpolation against directly summed gated linear attention);
 * a gate of 0 as a state reset.
 * Parity unpinned beyond those: the paper prints no output values of the layer.
 *
 * Layouts (row-major, all double):
 *   q,k [B,T,H,d_k]; v,y [B,T,H,d_v]; gate, lambda, fro [B,T,H];
 *   H state [B,H,d_k,d_k]; U state [B,H,d_v,d_k]  (U = sum v k^T).
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>

#define GKA_ORACLE_SOLVER_CHEBYSHEV 0
#define GKA_ORACLE_SOLVER_CHOLESKY 1

/* Weight schedule of Algorithm 1: omega_0 = 2, omega_i = 4 / (4 - rho^2 omega_{i-1}),
 * rho = (L - mu) / (L + mu).  Writes omega_0..omega_r (r + 1 values). */
void gka_oracle_omega_schedule(double L, double mu, int r, double *omega_out)
{
    double rho = (L - mu) / (L + mu);
    double omega = 2.0;
    omega_out[0] = omega;
    for (int i = 1; i <= r; ++i) {
        omega = 4.0 / (4.0 - rho * rho * omega);
        omega_out[i] = omega;
    }
}

/* Chebyshev Iteration (Algorithm 1) for A xi = q, A a D x D symmetric positive definite matrix (already
 * regularised) with spectrum inside [mu, L], written as the three-term semi-iterative method it is: with the
 * damped Richardson map
 *     R(x) = x + tau (q - A x),   tau = 2 / (L + mu),
 * the iterates are xi_0 = R(0) and xi_i = xi_{i-2} + omega_i (R(xi_{i-1}) - xi_{i-2}), omega_i from
 * gka_oracle_omega_schedule. (Substituting the first assignment of the algorithm's loop body into the second gives
 * exactly this.) r >= 0 passes; work holds 3*D doubles. */
static void richardson_map(int D, const double *A, const double *q, double tau, const double *x, double *out)
{
    for (int a = 0; a < D; ++a) {
        double Ax = 0.0;
        for (int b = 0; b < D; ++b) Ax += A[(size_t)a * D + b] * x[b];
        out[a] = x[a] + tau * (q[a] - Ax);
    }
}

void gka_oracle_chebyshev(int D, const double *A, const double *q, double L, double mu,
                          int r, double *xi_out, double *work)
{
    double *older = work;            /* xi_{i-2} */
    double *newer = work + D;        /* xi_{i-1} */
    double *mapped = work + 2 * D;   /* R(xi_{i-1}), then xi_i */
    const double tau = 2.0 / (L + mu);
    const double rho = (L - mu) / (L + mu);
    double omega = 2.0;
    memset(older, 0, (size_t)D * sizeof(double));
    richardson_map(D, A, q, tau, older, newer);
    for (int i = 1; i <= r; ++i) {
        omega = 4.0 / (4.0 - rho * rho * omega);
        richardson_map(D, A, q, tau, newer, mapped);
        for (int a = 0; a < D; ++a) mapped[a] = older[a] + omega * (mapped[a] - older[a]);
        double *recycled = older;
        older = newer;
        newer = mapped;
        mapped = recycled;
    }
    memcpy(xi_out, newer, (size_t)D * sizeof(double));
}

/* Exact solve of A x = q by Cholesky factorisation A = R^T R (A is overwritten).
 * Returns 0 on success, 1 if A is not positive definite. */
int gka_oracle_cholesky_solve(int D, double *A, const double *q, double *x)
{
    for (int j = 0; j < D; ++j) {
        double s = A[(size_t)j * D + j];
        for (int p = 0; p < j; ++p) s -= A[(size_t)p * D + j] * A[(size_t)p * D + j];
        if (!(s > 0.0)) return 1;
        double rjj = sqrt(s);
        A[(size_t)j * D + j] = rjj;
        for (int c = j + 1; c < D; ++c) {
            double u = A[(size_t)j * D + c];
            for (int p = 0; p < j; ++p) u -= A[(size_t)p * D + j] * A[(size_t)p * D + c];
            A[(size_t)j * D + c] = u / rjj;
        }
    }
    /* R^T z = q */
    for (int i = 0; i < D; ++i) {
        double s = q[i];
        for (int p = 0; p < i; ++p) s -= A[(size_t)p * D + i] * x[p];
        x[i] = s / A[(size_t)i * D + i];
    }
    /* R x = z */
    for (int i = D - 1; i >= 0; --i) {
        double s = x[i];
        for (int p = i + 1; p < D; ++p) s -= A[(size_t)i * D + p] * x[p];
        x[i] = s / A[(size_t)i * D + i];
    }
    return 0;
}

/* One token of Eq. (CH) on the explicit state of one pair.  Hs (d_k x d_k) and Us
 * (d_v x d_k) are updated in place.  lambda_given < 0 selects lambda = a * ||H_t||_F.
 * beta is the write gate of the beta-augmented variant (Remark in Section 4.1); beta = 1 is
 * the recurrence studied in the paper.  alpha is the alpha-connection of Section 4.3: the
 * readout is applied to the convex combination alpha * xhat_t + (1 - alpha) * q_t; alpha = 1
 * is Eq. (CH) as printed.  scratch holds d_k*d_k + 4*d_k doubles. */
static int token_step(int d_k, int d_v, double *Hs, double *Us, double gamma, double beta, double alpha,
                      const double *k, const double *v, const double *q,
                      double lambda_given, double a, int n_iter, int solver,
                      double *y, double *fro_out, double *xhat_out, double *scratch)
{
    double *A = scratch;
    double *xi = scratch + (size_t)d_k * d_k;
    double *work = xi + d_k;
    double fro2 = 0.0;
    for (int i = 0; i < d_k; ++i)
        for (int j = 0; j < d_k; ++j) {
            double h = gamma * Hs[(size_t)i * d_k + j] + beta * k[i] * k[j];
            Hs[(size_t)i * d_k + j] = h;
            fro2 += h * h;
        }
    for (int i = 0; i < d_v; ++i)
        for (int j = 0; j < d_k; ++j)
            Us[(size_t)i * d_k + j] = gamma * Us[(size_t)i * d_k + j] + beta * v[i] * k[j];
    double fro = sqrt(fro2);
    double lambda = (lambda_given >= 0.0) ? lambda_given : a * fro;
    double L = fro + lambda;
    double mu = lambda;
    for (int i = 0; i < d_k; ++i)
        for (int j = 0; j < d_k; ++j)
            A[(size_t)i * d_k + j] = Hs[(size_t)i * d_k + j] + (i == j ? lambda : 0.0);
    int rc = 0;
    if (solver == GKA_ORACLE_SOLVER_CHOLESKY)
        rc = gka_oracle_cholesky_solve(d_k, A, q, xi);
    else
        gka_oracle_chebyshev(d_k, A, q, L, mu, n_iter, xi, work);
    if (xhat_out) for (int j = 0; j < d_k; ++j) xhat_out[j] = xi[j];
    for (int j = 0; j < d_k; ++j) xi[j] = alpha * xi[j] + (1.0 - alpha) * q[j];
    for (int i = 0; i < d_v; ++i) {
        double s = 0.0;
        for (int j = 0; j < d_k; ++j) s += Us[(size_t)i * d_k + j] * xi[j];
        y[i] = s;
    }
    if (fro_out) *fro_out = fro;
    return rc;
}

/* Whole-sequence forward.  lambda may be NULL (then lambda_t = lambda_scale * ||H_t||_F);
 * beta, alpha (NULL = 1), H_init, U_init, H_final, U_final, fro_out, xhat_out may each be NULL.
 * Returns 0, or 1 if a Cholesky factorisation failed, or 2 on allocation failure. */
int gka_oracle_forward(int B, int T, int H, int d_k, int d_v,
                       const double *q, const double *k, const double *v,
                       const double *gate, const double *lambda, const double *beta, const double *alpha,
                       double lambda_scale, int n_iter, int solver,
                       const double *H_init, const double *U_init,
                       double *y, double *H_final, double *U_final,
                       double *fro_out, double *xhat_out)
{
    int status = 0;
    long npairs = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < npairs; ++p) {
        int b = (int)(p / H), h = (int)(p % H);
        size_t hh = (size_t)d_k * d_k, uu = (size_t)d_v * d_k;
        double *Hs = (double *)malloc(hh * sizeof(double));
        double *Us = (double *)malloc(uu * sizeof(double));
        double *scratch = (double *)malloc((hh + 4 * (size_t)d_k) * sizeof(double));
        if (!Hs || !Us || !scratch) {
#pragma omp critical
            status = 2;
            free(Hs); free(Us); free(scratch);
            continue;
        }
        if (H_init) memcpy(Hs, H_init + (size_t)p * hh, hh * sizeof(double));
        else memset(Hs, 0, hh * sizeof(double));
        if (U_init) memcpy(Us, U_init + (size_t)p * uu, uu * sizeof(double));
        else memset(Us, 0, uu * sizeof(double));
        for (int t = 0; t < T; ++t) {
            size_t tok = ((size_t)b * T + t) * H + h;
            int rc = token_step(d_k, d_v, Hs, Us, gate[tok], beta ? beta[tok] : 1.0, alpha ? alpha[tok] : 1.0,
                                k + tok * d_k, v + tok * d_v, q + tok * d_k,
                                lambda ? lambda[tok] : -1.0, lambda_scale, n_iter, solver,
                                y + tok * d_v, fro_out ? fro_out + tok : NULL,
                                xhat_out ? xhat_out + tok * d_k : NULL, scratch);
            if (rc) {
#pragma omp critical
                status = 1;
            }
        }
        if (H_final) memcpy(H_final + (size_t)p * hh, Hs, hh * sizeof(double));
        if (U_final) memcpy(U_final + (size_t)p * uu, Us, uu * sizeof(double));
        free(Hs); free(Us); free(scratch);
    }
    return status;
}

/* One recurrent decode step: one t-iteration of the loop above on stored states, which are
 * updated in place.  q,k [B,H,d_k]; v,y [B,H,d_v]; gate, lambda, fro [B,H]. */
int gka_oracle_decode_step(int B, int H, int d_k, int d_v,
                           double *H_state, double *U_state,
                           const double *q, const double *k, const double *v,
                           const double *gate, const double *lambda, const double *beta, const double *alpha,
                           double lambda_scale, int n_iter, int solver,
                           double *y, double *fro_out)
{
    int status = 0;
    long npairs = (long)B * H;
#pragma omp parallel for schedule(dynamic, 1)
    for (long p = 0; p < npairs; ++p) {
        size_t hh = (size_t)d_k * d_k, uu = (size_t)d_v * d_k;
        double *scratch = (double *)malloc((hh + 4 * (size_t)d_k) * sizeof(double));
        if (!scratch) {
#pragma omp critical
            status = 2;
            continue;
        }
        int rc = token_step(d_k, d_v, H_state + (size_t)p * hh, U_state + (size_t)p * uu,
                            gate[p], beta ? beta[p] : 1.0, alpha ? alpha[p] : 1.0,
                            k + (size_t)p * d_k, v + (size_t)p * d_v, q + (size_t)p * d_k,
                            lambda ? lambda[p] : -1.0, lambda_scale, n_iter, solver,
                            y + (size_t)p * d_v, fro_out ? fro_out + p : NULL, NULL, scratch);
        if (rc) {
#pragma omp critical
            status = 1;
        }
        free(scratch);
    }
    return status;
}

int gka_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}
