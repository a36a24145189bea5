/*
 * Reference ("oracle") for the table-interpolated variant of the Chebyshev-KAN
 * layer, fp64, CPU.  TEST INFRASTRUCTURE, like chebykan_oracle.c: plain, slow,
 * written from the paper's description, sharing nothing with the GPU path.
 *
 * The variant (paper Sec. 4.2, "Polynomial Operators Acceleration via LUT"):
 *
 *   offline   LUT[k][i] = T_k(x_i),  x_i = -1 + i*Delta,  Delta = 2/(n-1),
 *             i = 0..n-1, T_k by the recurrence of Eq. 2           (Sec. 4.2.1)
 *   online    u   = tanh(x)
 *             pos = (u+1)/2 * (n-1),  c = floor(pos),  f = pos - c
 *             T_k(u)  ~ LUT[k][c] + f * (LUT[k][c+1] - LUT[k][c])   (Sec. 4.2.2)
 *             T_k'(u) ~ (LUT[k][c+1] - LUT[k][c]) / Delta           (difference of
 *                        neighbouring samples, Sec. 4.2.2 last paragraph)
 *   layer     y, dC, dx exactly as in the exact layer (Alg. 1, Alg. 2) with these
 *             two approximations in place of T_k and T_k'.
 *
 * Readings taken: at u = +1 pos = n-1 and sample c+1 would not exist, so c is
 * clamped to n-2 (then f = 1 and the value is LUT[k][n-1]); dx includes the tanh
 * derivative (1-u^2) as in the exact layer; rows k = 0 and 1 of the table are
 * interpolated like every other row.  The table is an INPUT here (double
 * values, normally the fp32-rounded table the GPU also receives), so both sides
 * interpolate the same numbers; oracle_lut_build is the fp64 construction.
 *
 * `shift` (optional, per input element) is added to the cell index c before
 * interpolating; the line of the neighbouring cell is then evaluated at the same
 * pos.  Tests use it for elements whose pos lies within rounding distance of a
 * cell boundary, where an fp32 implementation may legitimately pick the other
 * cell: T is continuous across the boundary, the difference quotient is not.
 *
 * Second-order derivative ("auxiliary table", the other option Sec. 4.2.2 names for the
 * derivative).  Reading taken: the auxiliary table holds samples of the derivative itself,
 *   dLUT[k][i] = T_k'(x_i) = k U_{k-1}(x_i)   (second-kind recurrence, finite at x = +-1),
 * and is interpolated exactly like the value table,
 *   T_k'(u) ~ dLUT[k][c] + f * (dLUT[k][c+1] - dLUT[k][c]),
 * which is second-order in Delta (error <= Delta^2/8 max|T_k'''|,  max|T_k'''| =
 * k^2 (k^2-1)(k^2-4)/15 at x = +-1) and continuous across knots.  A table of pre-computed
 * neighbour differences would reproduce the first-order quotient above bit for bit and is
 * therefore not a separate variant.  oracle_dx_lut2 is the dx of oracle_backward_lut with this
 * derivative; dC does not involve the derivative and is unchanged.
 *
 * Pins (tests/test_oracle_lut_pins.py): table against cos(k acos x); exactness
 * at grid points and for degree <= 1; |T_lut - T| <= Delta^2/8 * max|T_k''|;
 * the difference quotient equals T_k' somewhere inside the cell; dx is the
 * numerical derivative of the interpolated forward inside a cell; adjoint
 * identity <dy,y> = <C,dC>; convergence to the exact layer as n grows.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>

#define LUT_ORACLE_MAX_DEGREE 64

int oracle_lut_build(double *lut, int d, int64_t n)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
    const double delta = 2.0 / (double)(n - 1);
    for (int64_t i = 0; i < n; ++i) {
        /* the last point is set exactly so that rounding in i*delta cannot leave [-1,1] */
        const double xi = (i == n - 1) ? 1.0 : -1.0 + (double)i * delta;
        double t_prev = 1.0, t_cur = xi;
        lut[0 * n + i] = 1.0;
        if (d >= 1) lut[1 * n + i] = xi;
        for (int k = 1; k < d; ++k) {
            const double t_next = 2.0 * xi * t_cur - t_prev;
            lut[(int64_t)(k + 1) * n + i] = t_next;
            t_prev = t_cur;
            t_cur = t_next;
        }
    }
    return 0;
}

/* dLUT[k][i] = T_k'(x_i) on the same grid, T_k' = k U_{k-1} with U_0 = 1, U_1 = 2x, U_{j+1} = 2x U_j - U_{j-1}. */
int oracle_lut_build_derivative(double *dlut, int d, int64_t n)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
    const double delta = 2.0 / (double)(n - 1);
    for (int64_t i = 0; i < n; ++i) {
        const double xi = (i == n - 1) ? 1.0 : -1.0 + (double)i * delta;
        double u_prev = 0.0, u_cur = 1.0;   /* U_{-1} = 0, U_0 = 1 */
        dlut[0 * n + i] = 0.0;
        for (int k = 1; k <= d; ++k) {
            dlut[(int64_t)k * n + i] = (double)k * u_cur;     /* k U_{k-1} */
            const double u_next = 2.0 * xi * u_cur - u_prev;
            u_prev = u_cur;
            u_cur = u_next;
        }
    }
    return 0;
}

/* Interpolated derivative table at u: dT[k] = dLUT[k][c] + f (dLUT[k][c+1] - dLUT[k][c]), same cell rule. */
void oracle_lut_eval_derivative(const double *dlut, int d, int64_t n, double u, double *dT)
{
    const double pos = (u + 1.0) / 2.0 * (double)(n - 1);
    int64_t c = (int64_t)floor(pos);
    if (c > n - 2) c = n - 2;
    if (c < 0) c = 0;
    const double f = pos - (double)c;
    for (int k = 0; k <= d; ++k) {
        const double lo = dlut[(int64_t)k * n + c], hi = dlut[(int64_t)k * n + c + 1];
        dT[k] = lo + f * (hi - lo);
    }
}

/* Interpolated T_0..T_d and difference quotients dT_0..dT_d at u in [-1,1]. */
void oracle_lut_eval(const double *lut, int d, int64_t n, double u, int shift,
                     double *T, double *dT, int64_t *cell, double *frac)
{
    const double delta = 2.0 / (double)(n - 1);
    const double pos = (u + 1.0) / 2.0 * (double)(n - 1);
    int64_t c = (int64_t)floor(pos);
    if (c > n - 2) c = n - 2;
    if (c < 0) c = 0;
    if (cell) *cell = c;
    if (frac) *frac = pos - (double)c;
    c += shift;
    if (c > n - 2) c = n - 2;
    if (c < 0) c = 0;
    const double f = pos - (double)c;
    for (int k = 0; k <= d; ++k) {
        const double lo = lut[(int64_t)k * n + c], hi = lut[(int64_t)k * n + c + 1];
        if (T) T[k] = lo + f * (hi - lo);
        if (dT) dT[k] = (hi - lo) / delta;
    }
}

int oracle_forward_lut(const double *x, const double *C, const double *lut, int64_t n, double *y,
                       int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double T[LUT_ORACLE_MAX_DEGREE + 1];
        for (int64_t o = 0; o < O; ++o) y[b * O + o] = 0.0;
        for (int64_t i = 0; i < I; ++i) {
            const double u = tanh(x[b * I + i]);
            oracle_lut_eval(lut, d, n, u, 0, T, NULL, NULL, NULL);
            for (int64_t o = 0; o < O; ++o) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k) acc += C[(i * O + o) * K + k] * T[k];
                y[b * O + o] += acc;
            }
        }
    }
    return 0;
}

/* dx (skipped when NULL), dC (skipped when NULL); shift: [B,I] or NULL; frac_out: [B,I] or NULL. */
int oracle_backward_lut(const double *x, const double *C, const double *dy, const double *lut, int64_t n,
                        const int8_t *shift, double *dx, double *dC, double *frac_out,
                        int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
    const int64_t K = d + 1;
    if (dx || frac_out) {
#pragma omp parallel for schedule(static)
        for (int64_t b = 0; b < B; ++b) {
            double dT[LUT_ORACLE_MAX_DEGREE + 1];
            for (int64_t i = 0; i < I; ++i) {
                const double u = tanh(x[b * I + i]);
                double f;
                oracle_lut_eval(lut, d, n, u, shift ? shift[b * I + i] : 0, NULL, dT, NULL, &f);
                if (frac_out) frac_out[b * I + i] = f;
                if (!dx) continue;
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
            double T[LUT_ORACLE_MAX_DEGREE + 1];
            for (int64_t e = 0; e < O * K; ++e) dC[i * O * K + e] = 0.0;
            for (int64_t b = 0; b < B; ++b) {
                const double u = tanh(x[b * I + i]);
                oracle_lut_eval(lut, d, n, u, 0, T, NULL, NULL, NULL);
                for (int64_t o = 0; o < O; ++o) {
                    const double g = dy[b * O + o];
                    for (int64_t k = 0; k < K; ++k) dC[(i * O + o) * K + k] += T[k] * g;
                }
            }
        }
    }
    return 0;
}

/* dx of the layer with the interpolated derivative table in place of the difference quotient. */
int oracle_dx_lut2(const double *x, const double *C, const double *dy, const double *dlut, int64_t n, double *dx,
                   int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
    const int64_t K = d + 1;
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {
        double dT[LUT_ORACLE_MAX_DEGREE + 1];
        for (int64_t i = 0; i < I; ++i) {
            const double u = tanh(x[b * I + i]);
            oracle_lut_eval_derivative(dlut, d, n, u, dT);
            double acc = 0.0;
            for (int64_t o = 0; o < O; ++o) {
                double inner = 0.0;
                for (int64_t k = 1; k < K; ++k) inner += C[(i * O + o) * K + k] * dT[k];
                acc += dy[b * O + o] * inner;
            }
            dx[b * I + i] = (1.0 - u * u) * acc;
        }
    }
    return 0;
}

/* Sampled coefficient gradients: out[s] = dC[is[s], os[s], ks[s]] of the interpolated layer,
 * one requested element at a time (for spot checks of full-size results). */
int oracle_dC_lut_at(const double *x, const double *dy, const double *lut, int64_t n,
                     const int64_t *is, const int64_t *os, const int64_t *ks, int64_t count, double *out,
                     int64_t B, int64_t I, int64_t O, int d)
{
    if (d < 0 || d > LUT_ORACLE_MAX_DEGREE || n < 2) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t s = 0; s < count; ++s) {
        double T[LUT_ORACLE_MAX_DEGREE + 1];
        double acc = 0.0;
        for (int64_t b = 0; b < B; ++b) {
            oracle_lut_eval(lut, d, n, tanh(x[b * I + is[s]]), 0, T, NULL, NULL, NULL);
            acc += T[ks[s]] * dy[b * O + os[s]];
        }
        out[s] = acc;
    }
    return 0;
}
