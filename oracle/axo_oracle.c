/*
 * CPU oracle for one GPU's share of a 3D-tensor-parallel fully-connected layer.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
 * the shard GEMMs compute.  It shares no code with the HIP library and must never
 * be called from the product path; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg use it.
 *
 * What it states (paper Section 3.2, "serial computation in an FC layer", and
 * Algorithm 1, local products of the forward and backward functions):
 *
 *   forward   O  = I  x W            Y [t,n] = sum_k X [t,k] * W[k,n]
 *   dgrad     dI = dO x W^T          dX[t,k] = sum_n dY[t,n] * W[k,n]
 *   wgrad     dW = I^T x dO          dW[k,n] = sum_t X [t,k] * dY[t,n]
 *
 * with I = X [M x Kl], W [Kl x Nl], O = Y [M x Nl] the local row-major blocks
 * (Figure 1 fixes I in R^{m x k}, W in R^{k x n}).  Inputs are bf16 bit patterns,
 * widened exactly to fp64; every sum runs in fp64 in ascending index order; the
 * result stays fp64 (no rounding to bf16).  The optional epilogue (bias add, GELU)
 * is not in the paper; it is the usual GPT MLP epilogue and is evaluated in fp64
 * with libm on the fp64 sum.
 *
 * The steps either side of the three products in a real layer (not in the paper's Algorithm 1,
 * which stops at the products; Section 6.1 trains in mixed precision): the GELU derivative
 * applied to the data gradient, the bias gradient (column sums of dO) and the accumulation of
 * the weight gradient into an fp32 buffer are stated here too, in fp64.
 *
 * Every routine takes an optional list of output rows, so that at full benchmark
 * sizes a sample of whole output rows can be computed one by one.
 *
 * Parity pins (tests, not here): brute-force long-double loops on tiny shapes,
 * numpy fp64 matmul, the decomposition identity of Section 3.2 / Algorithm 1,
 * the adjoint identity, GELU invariants, structured inputs with exact answers.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_EPI_NONE 0
#define ORACLE_EPI_BIAS 1
#define ORACLE_EPI_BIAS_GELU_TANH 2
#define ORACLE_EPI_BIAS_GELU_ERF 3

static inline double widen(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* GELU, exact form: x * Phi(x) with Phi the standard normal CDF. */
double oracle_gelu_erf(double x)
{
    return 0.5 * x * (1.0 + erf(x * 0.70710678118654752440));
}

/* GELU, tanh form (Hendrycks & Gimpel): 0.5 x (1 + tanh( sqrt(2/pi) (x + 0.044715 x^3) )). */
double oracle_gelu_tanh(double x)
{
    const double c = 0.79788456080286535588; /* sqrt(2/pi) */
    return 0.5 * x * (1.0 + tanh(c * (x + 0.044715 * x * x * x)));
}

/* d/dx of the exact GELU:  Phi(x) + x phi(x)  (phi, Phi: standard normal density and CDF). */
double oracle_dgelu_erf(double x)
{
    const double phi = 0.39894228040143267794 * exp(-0.5 * x * x); /* 1/sqrt(2 pi) */
    return 0.5 * (1.0 + erf(x * 0.70710678118654752440)) + x * phi;
}

/* d/dx of the tanh-form GELU: with u = c (x + a x^3), 0.5 (1 + tanh u) + 0.5 x (1 - tanh^2 u) c (1 + 3 a x^2). */
double oracle_dgelu_tanh(double x)
{
    const double c = 0.79788456080286535588, a = 0.044715;
    const double th = tanh(c * (x + a * x * x * x));
    return 0.5 * (1.0 + th) + 0.5 * x * (1.0 - th * th) * c * (1.0 + 3.0 * a * x * x);
}

/* Forward local product (Algorithm 1, forward function, the local multiply).
 * out[r, n] for r in rows (or all M rows when rows == NULL); out is [n_rows x Nl], dense.
 * bias is [Nl] bf16 bits or NULL. */
int oracle_fc_fwd(const uint16_t *X, int64_t ldx, const uint16_t *W, int64_t ldw,
                  const uint16_t *bias, int epilogue, int64_t M, int64_t Kl, int64_t Nl,
                  const int64_t *rows, int64_t n_rows, double *out)
{
    if (rows == NULL) n_rows = M;
    if (epilogue != ORACLE_EPI_NONE && bias == NULL) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t t = rows ? rows[r] : r;
        double *y = out + r * Nl;
        for (int64_t n = 0; n < Nl; ++n) y[n] = 0.0;
        for (int64_t k = 0; k < Kl; ++k) {
            const double x = widen(X[t * ldx + k]);
            const uint16_t *w = W + k * ldw;
            for (int64_t n = 0; n < Nl; ++n) y[n] += x * widen(w[n]);
        }
        if (epilogue != ORACLE_EPI_NONE) {
            for (int64_t n = 0; n < Nl; ++n) {
                double v = y[n] + widen(bias[n]);
                if (epilogue == ORACLE_EPI_BIAS_GELU_TANH) v = oracle_gelu_tanh(v);
                else if (epilogue == ORACLE_EPI_BIAS_GELU_ERF) v = oracle_gelu_erf(v);
                y[n] = v;
            }
        }
    }
    return 0;
}

/* Backward data-gradient local product (Algorithm 1, backward function, dO x W^T).
 * out[r, k] = sum_n dY[t_r, n] * W[k, n];  out is [n_rows x Kl]. */
int oracle_fc_dgrad(const uint16_t *dY, int64_t lddy, const uint16_t *W, int64_t ldw,
                    int64_t M, int64_t Kl, int64_t Nl,
                    const int64_t *rows, int64_t n_rows, double *out)
{
    if (rows == NULL) n_rows = M;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t t = rows ? rows[r] : r;
        const uint16_t *g = dY + t * lddy;
        for (int64_t k = 0; k < Kl; ++k) {
            const uint16_t *w = W + k * ldw;
            double s = 0.0;
            for (int64_t n = 0; n < Nl; ++n) s += widen(g[n]) * widen(w[n]);
            out[r * Kl + k] = s;
        }
    }
    return 0;
}

/* Data gradient through an activation: out[r, k] = (sum_n dY[t_r, n] W[k, n]) * act'(P[t_r, k]),
 * P the bf16 pre-activation of the layer below; act: ORACLE_EPI_BIAS_GELU_TANH or _ERF. */
int oracle_fc_dgrad_act(const uint16_t *dY, int64_t lddy, const uint16_t *W, int64_t ldw,
                        const uint16_t *P, int64_t ldp, int act, int64_t M, int64_t Kl, int64_t Nl,
                        const int64_t *rows, int64_t n_rows, double *out)
{
    if (act != ORACLE_EPI_BIAS_GELU_TANH && act != ORACLE_EPI_BIAS_GELU_ERF) return -1;
    int rc = oracle_fc_dgrad(dY, lddy, W, ldw, M, Kl, Nl, rows, n_rows, out);
    if (rc) return rc;
    if (rows == NULL) n_rows = M;
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t t = rows ? rows[r] : r;
        for (int64_t k = 0; k < Kl; ++k) {
            const double p = widen(P[t * ldp + k]);
            out[r * Kl + k] *= act == ORACLE_EPI_BIAS_GELU_TANH ? oracle_dgelu_tanh(p) : oracle_dgelu_erf(p);
        }
    }
    return 0;
}

/* Bias gradient: out[n] = sum_t dY[t, n]  (the column sums of dO), ascending t. */
int oracle_bias_grad(const uint16_t *dY, int64_t lddy, int64_t M, int64_t Nl, double *out)
{
    for (int64_t n = 0; n < Nl; ++n) out[n] = 0.0;
    for (int64_t t = 0; t < M; ++t)
        for (int64_t n = 0; n < Nl; ++n) out[n] += widen(dY[t * lddy + n]);
    return 0;
}

/* Backward weight-gradient local product (Algorithm 1, backward function, I^T x dO).
 * out[r, n] = sum_t X[t, k_r] * dY[t, n];  rows index the Kl rows of dW; out is [n_rows x Nl]. */
int oracle_fc_wgrad(const uint16_t *X, int64_t ldx, const uint16_t *dY, int64_t lddy,
                    int64_t M, int64_t Kl, int64_t Nl,
                    const int64_t *rows, int64_t n_rows, double *out)
{
    if (rows == NULL) n_rows = Kl;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t k = rows ? rows[r] : r;
        double *d = out + r * Nl;
        for (int64_t n = 0; n < Nl; ++n) d[n] = 0.0;
        for (int64_t t = 0; t < M; ++t) {
            const double x = widen(X[t * ldx + k]);
            const uint16_t *g = dY + t * lddy;
            for (int64_t n = 0; n < Nl; ++n) d[n] += x * widen(g[n]);
        }
    }
    return 0;
}

/* Comparison metrics between a candidate (bf16 bits, leading dimension ldc) and the fp64
 * oracle block [rows x cols]:
 *   res[0] = ||C - O||_F / ||O||_F            (0 when both norms are 0)
 *   res[1] = max over elements of |C - O| / max_c |O[r, c]|   (rows with zero max: abs error)
 *   res[2] = number of elements with |C - O| > per_elem_tol * max_c |O[r, c]|
 *   res[3] = number of non-finite candidate elements                                    */
int oracle_compare_bf16(const uint16_t *C, int64_t ldc, const double *O, int64_t rows, int64_t cols,
                        double per_elem_tol, double *res)
{
    double num = 0.0, den = 0.0, worst = 0.0, nbad = 0.0, nnan = 0.0;
    for (int64_t r = 0; r < rows; ++r) {
        double rmax = 0.0;
        for (int64_t c = 0; c < cols; ++c) {
            double a = fabs(O[r * cols + c]);
            if (a > rmax) rmax = a;
        }
        for (int64_t c = 0; c < cols; ++c) {
            double g = widen(C[r * ldc + c]);
            double o = O[r * cols + c];
            if (!isfinite(g)) { nnan += 1.0; continue; }
            double e = fabs(g - o);
            num += e * e;
            den += o * o;
            double rel = rmax > 0.0 ? e / rmax : e;
            if (rel > worst) worst = rel;
            if (e > per_elem_tol * rmax) nbad += 1.0;
        }
    }
    res[0] = den > 0.0 ? sqrt(num / den) : (num > 0.0 ? INFINITY : 0.0);
    res[1] = worst;
    res[2] = nbad;
    res[3] = nnan;
    return 0;
}
