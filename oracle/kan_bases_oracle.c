/*
 * Reference ("oracle") for KAN layers on other polynomial / trigonometric bases, fp64, CPU.
 * TEST INFRASTRUCTURE, like chebykan_oracle.c: plain, slow, independent of the GPU path.
 *
 * The paper (Sec. 2.3, "The characteristics of the KAN variants") observes that Legendre,
 * Hermite and Fourier KANs share the layer's skeleton - expand each input into K basis
 * functions by a short recurrence  alpha_k B_{k+1} = beta_k(x) B_k - gamma_k B_{k-1},
 * contract with learnable coefficients - and Sec. 6.3 reports the method applied to them.
 * It gives no formulas for these bases; the textbook definitions are taken:
 *
 *   kind 1  Legendre on u = tanh(x):   (k+1) P_{k+1} = (2k+1) u P_k - k P_{k-1},  P_0 = 1, P_1 = u
 *                                       P'_{k+1} = P'_{k-1} + (2k+1) P_k
 *   kind 2  Hermite (physicists') on u = tanh(x):  H_{k+1} = 2 u H_k - 2k H_{k-1},  H_0 = 1, H_1 = 2u
 *                                       H'_k = 2k H_{k-1}
 *   kind 3  Fourier on the raw input x, "degree" d = 2G:
 *                                       B_0 = 1, B_{2m-1} = cos(m x), B_{2m} = sin(m x), m = 1..G
 *                                       (the constant B_0 keeps the skeleton's K = d+1 functions)
 *
 * and the layer is the one of chebykan_oracle.c with B_k in place of T_k:
 *   y[b,o]    = sum_i sum_k C[i,o,k] B_k(x[b,i])
 *   dC[i,o,k] = sum_b B_k(x[b,i]) dy[b,o]
 *   dx[b,i]   = sum_o dy[b,o] sum_k C[i,o,k] dB_k/dx,  dB_k/dx = (1-u^2) B_k'(u) for kinds 1, 2
 *
 * kind 0 is the Chebyshev layer itself (by Eq. 2), so that the generic code path can be
 * checked against chebykan_oracle.c.
 *
 * Pins (tests/test_oracle_bases_pins.py): numpy's Legendre / Hermite bases and derivatives,
 * explicit low-degree polynomials, end-point values, direct cos/sin, finite differences of
 * the layer, the adjoint identity, kind 0 against the Chebyshev oracle.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define BASES_MAX_DEGREE 64

/* B_0..B_d and dB_0/dx..dB_d/dx at input x (x is the RAW layer input). */
int oracle_basis_eval(int kind, double x, int d, double *Bv, double *dB)
{
    if (d < 0 || d > BASES_MAX_DEGREE) return -1;
    if (kind == 3) {
        if (d % 2 != 0) return -1;
        Bv[0] = 1.0;
        dB[0] = 0.0;
        for (int m = 1; m <= d / 2; ++m) {
            const double c = cos((double)m * x), s = sin((double)m * x);
            Bv[2 * m - 1] = c;
            Bv[2 * m] = s;
            dB[2 * m - 1] = -(double)m * s;
            dB[2 * m] = (double)m * c;
        }
        return 0;
    }
    const double u = tanh(x);
    const double chain = 1.0 - u * u;
    double D[BASES_MAX_DEGREE + 1]; /* derivative with respect to u */
    Bv[0] = 1.0;
    D[0] = 0.0;
    if (kind == 0) { /* Chebyshev: T and T' = k U_{k-1} */
        if (d >= 1) Bv[1] = u;
        for (int k = 1; k < d; ++k) Bv[k + 1] = 2.0 * u * Bv[k] - Bv[k - 1];
        double U_prev = 0.0, U_cur = 1.0;
        for (int k = 1; k <= d; ++k) {
            D[k] = (double)k * U_cur;
            const double U_next = 2.0 * u * U_cur - U_prev;
            U_prev = U_cur;
            U_cur = U_next;
        }
    } else if (kind == 1) { /* Legendre */
        if (d >= 1) { Bv[1] = u; D[1] = 1.0; }
        for (int k = 1; k < d; ++k) {
            Bv[k + 1] = ((double)(2 * k + 1) * u * Bv[k] - (double)k * Bv[k - 1]) / (double)(k + 1);
            D[k + 1] = D[k - 1] + (double)(2 * k + 1) * Bv[k];
        }
    } else if (kind == 2) { /* Hermite, physicists' */
        if (d >= 1) { Bv[1] = 2.0 * u; D[1] = 2.0; }
        for (int k = 1; k < d; ++k) {
            Bv[k + 1] = 2.0 * u * Bv[k] - 2.0 * (double)k * Bv[k - 1];
            D[k + 1] = 2.0 * (double)(k + 1) * Bv[k];
        }
    } else {
        return -1;
    }
    for (int k = 0; k <= d; ++k) dB[k] = chain * D[k];
    return 0;
}

int oracle_forward_basis(int kind, const double *x, const double *C, double *y,
                         int64_t B, int64_t I, int64_t O, int d)
{
    double probe_B[BASES_MAX_DEGREE + 1], probe_d[BASES_MAX_DEGREE + 1];
    if (oracle_basis_eval(kind, 0.0, d, probe_B, probe_d) != 0) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double Bv[BASES_MAX_DEGREE + 1], dB[BASES_MAX_DEGREE + 1];
        for (int64_t o = 0; o < O; ++o) y[b * O + o] = 0.0;
        for (int64_t i = 0; i < I; ++i) {
            oracle_basis_eval(kind, x[b * I + i], d, Bv, dB);
            for (int64_t o = 0; o < O; ++o) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k) acc += C[(i * O + o) * K + k] * Bv[k];
                y[b * O + o] += acc;
            }
        }
    }
    return 0;
}

int oracle_backward_basis(int kind, const double *x, const double *C, const double *dy,
                          double *dx, double *dC, int64_t B, int64_t I, int64_t O, int d)
{
    double probe_B[BASES_MAX_DEGREE + 1], probe_d[BASES_MAX_DEGREE + 1];
    if (oracle_basis_eval(kind, 0.0, d, probe_B, probe_d) != 0) return -1;
    const int64_t K = d + 1;
    if (dx) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            double Bv[BASES_MAX_DEGREE + 1], dB[BASES_MAX_DEGREE + 1];
            for (int64_t i = 0; i < I; ++i) {
                oracle_basis_eval(kind, x[b * I + i], d, Bv, dB);
                double acc = 0.0;
                for (int64_t o = 0; o < O; ++o) {
                    double inner = 0.0;
                    for (int64_t k = 0; k < K; ++k) inner += C[(i * O + o) * K + k] * dB[k];
                    acc += dy[b * O + o] * inner;
                }
                dx[b * I + i] = acc;
            }
        }
    }
    if (dC) {
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < I; ++i) {
            double Bv[BASES_MAX_DEGREE + 1], dB[BASES_MAX_DEGREE + 1];
            for (int64_t e = 0; e < O * K; ++e) dC[i * O * K + e] = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                oracle_basis_eval(kind, x[b * I + i], d, Bv, dB);
                for (int64_t o = 0; o < O; ++o) {
                    const double g = dy[b * O + o];
                    for (int64_t k = 0; k < K; ++k) dC[(i * O + o) * K + k] += Bv[k] * g;
                }
            }
        }
    }
    return 0;
}
