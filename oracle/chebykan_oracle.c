/*
 * Reference ("oracle") implementation of one Chebyshev-KAN layer, fp64, CPU.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, index-order evaluation of
 * the layer's mathematical definition; it exists so that the GPU library can be
 * checked against something written independently of it.  It shares no code,
 * header, table or constant with the GPU path and must never be called from the
 * product path.  Only the tests, the smoke check and the benchmark's CPU
 * baseline leg use it.
 *
 * What is computed (paper: Sec. 2.2 Eq. 1-3, Fig. 3 caption, Alg. 1 inner loop,
 * Alg. 2 inner loops):
 *
 *   u[b,i]    = tanh(x[b,i])                                   (Fig. 3 caption)
 *   T_0 = 1, T_1 = u, T_{k+1} = 2 u T_k - T_{k-1}              (Eq. 2)
 *   y[b,o]    = sum_i sum_{k=0..d} C[i,o,k] T_k(u[b,i])        (Eq. 3 without bias)
 *   dC[i,o,k] = sum_b T_k(u[b,i]) dy[b,o]                      (Alg. 2, coeff_grad)
 *   dx[b,i]   = (1 - u^2) sum_o dy[b,o] sum_{k=1..d} C[i,o,k] T_k'(u)
 *                                                              (Alg. 2, x_grad, with
 *                                                               the chain rule through tanh)
 *   T_k'(u)   = k U_{k-1}(u),  U_0 = 1, U_1 = 2u, U_{k+1} = 2 u U_k - U_{k-1}
 *
 * Readings of the paper taken here: no bias term; the gradient is with respect
 * to the raw input x, so the tanh derivative (1-u^2) is included; the analytic
 * derivative is used, not a table difference; coefficients are laid out
 * [in][out][degree+1]; outputs are overwritten, not accumulated into.
 *
 * All inputs are double arrays (callers promote fp32 bits exactly), all
 * arithmetic and accumulation is double, loops run in index order.
 * OpenMP, when enabled, only distributes independent output elements.
 *
 * Every function here is pinned by tests against closed forms
 * (T_k(cos t) = cos(k t), explicit low-degree polynomials, T_k'(1) = k^2),
 * an independent library basis, brute force with the trigonometric form,
 * the adjoint identity <dy,y> = <C,dC> and central finite differences.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_MAX_DEGREE 64

/* T_0..T_d at u by the three-term recurrence (Eq. 2). */
void oracle_cheb_T(double u, int d, double *T)
{
    T[0] = 1.0;
    if (d >= 1) T[1] = u;
    for (int k = 1; k < d; ++k) T[k + 1] = 2.0 * u * T[k] - T[k - 1];
}

/* T_0..T_d at u by the trigonometric definition (Eq. 1); |u| <= 1. */
void oracle_cheb_T_trig(double u, int d, double *T)
{
    double theta = acos(u);
    for (int k = 0; k <= d; ++k) T[k] = cos((double)k * theta);
}

/* T'_0..T'_d at u:  T'_k = k U_{k-1}, U from its own three-term recurrence. */
void oracle_cheb_dT(double u, int d, double *dT)
{
    dT[0] = 0.0;
    double U_prev = 0.0; /* U_{-1} */
    double U_cur = 1.0;  /* U_0   */
    for (int k = 1; k <= d; ++k) {
        dT[k] = (double)k * U_cur;              /* k U_{k-1} */
        double U_next = 2.0 * u * U_cur - U_prev;
        U_prev = U_cur;
        U_cur = U_next;
    }
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* y[b,o] for every b,o.  x:[B,I]  C:[I,O,d+1]  y:[B,O], all row-major. */
int oracle_forward(const double *x, const double *C, double *y,
                   int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > ORACLE_MAX_DEGREE) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double T[ORACLE_MAX_DEGREE + 1];
        for (int64_t o = 0; o < O; ++o) y[b * O + o] = 0.0;
        for (int64_t i = 0; i < I; ++i) {
            double u = tanh(x[b * I + i]);
            oracle_cheb_T(u, d, T);
            for (int64_t o = 0; o < O; ++o) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k) acc += C[(i * O + o) * K + k] * T[k];
                y[b * O + o] += acc;
            }
        }
    }
    return 0;
}

/* dx[b,i] for every b,i (skipped when dx is NULL) and dC[i,o,k] for every
 * i,o,k (skipped when dC is NULL).  dy:[B,O]. */
int oracle_backward(const double *x, const double *C, const double *dy,
                    double *dx, double *dC,
                    int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > ORACLE_MAX_DEGREE) return -1;
    const int64_t K = d + 1;
    if (dx) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            double dT[ORACLE_MAX_DEGREE + 1];
            for (int64_t i = 0; i < I; ++i) {
                double u = tanh(x[b * I + i]);
                oracle_cheb_dT(u, d, dT);
                double acc = 0.0;
                for (int64_t o = 0; o < O; ++o) {
                    double inner = 0.0;
                    for (int64_t k = 1; k < K; ++k) inner += C[(i * O + o) * K + k] * dT[k];
                    acc += dy[b * O + o] * inner;
                }
                dx[b * I + i] = (1.0 - u * u) * acc;
            }
        }
    }
    if (dC) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < I; ++i) {
            double T[ORACLE_MAX_DEGREE + 1];
            for (int64_t e = 0; e < O * K; ++e) dC[i * O * K + e] = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                double u = tanh(x[b * I + i]);
                oracle_cheb_T(u, d, T);
                for (int64_t o = 0; o < O; ++o) {
                    double g = dy[b * O + o];
                    for (int64_t k = 0; k < K; ++k) dC[(i * O + o) * K + k] += T[k] * g;
                }
            }
        }
    }
    return 0;
}

/* Sampled outputs: the same definitions, one requested element at a time, so
 * that full-size GPU results can be spot-checked without the full CPU run. */
int oracle_forward_at(const double *x, const double *C,
                      const int64_t *bs, const int64_t *os, int64_t n, double *out,
                      int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > ORACLE_MAX_DEGREE) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n; ++s) {
        int64_t b = bs[s], o = os[s];
        double T[ORACLE_MAX_DEGREE + 1];
        double acc = 0.0;
        for (int64_t i = 0; i < I; ++i) {
            oracle_cheb_T(tanh(x[b * I + i]), d, T);
            for (int64_t k = 0; k < K; ++k) acc += C[(i * O + o) * K + k] * T[k];
        }
        out[s] = acc;
    }
    (void)B;
    return 0;
}

int oracle_dx_at(const double *x, const double *C, const double *dy,
                 const int64_t *bs, const int64_t *is, int64_t n, double *out,
                 int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > ORACLE_MAX_DEGREE) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n; ++s) {
        int64_t b = bs[s], i = is[s];
        double dT[ORACLE_MAX_DEGREE + 1];
        double u = tanh(x[b * I + i]);
        oracle_cheb_dT(u, d, dT);
        double acc = 0.0;
        for (int64_t o = 0; o < O; ++o) {
            double inner = 0.0;
            for (int64_t k = 1; k < K; ++k) inner += C[(i * O + o) * K + k] * dT[k];
            acc += dy[b * O + o] * inner;
        }
        out[s] = (1.0 - u * u) * acc;
    }
    (void)B;
    return 0;
}

int oracle_dC_at(const double *x, const double *dy,
                 const int64_t *is, const int64_t *os, const int64_t *ks, int64_t n, double *out,
                 int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > ORACLE_MAX_DEGREE) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < n; ++s) {
        int64_t i = is[s], o = os[s], k = ks[s];
        double T[ORACLE_MAX_DEGREE + 1];
        double acc = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            oracle_cheb_T(tanh(x[b * I + i]), d, T);
            acc += T[k] * dy[b * O + o];
        }
        out[s] = acc;
    }
    return 0;
}
