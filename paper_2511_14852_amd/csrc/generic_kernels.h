// Any-degree kernels: one thread per output element, exact recurrences, plain
// fp32 VALU arithmetic.  They serve degrees and shapes the MFMA kernels are not
// specialised for and give an on-device cross-check of those kernels.
//
// T_k is advanced in the difference form of the recurrence on w = 1 - |u| (see
// cheb_T_of_x), which holds its accuracy at any degree; odd k take the sign of x.
//
// Every reduction runs in a fixed order inside one thread, with the running sum
// folded into a second accumulator every FOLD terms so that long fp32 sums do
// not lose accuracy.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "basis.h"

namespace chebykan {

constexpr int GENERIC_FOLD = 16;

// y[b,o] = sum_i sum_k C[i,o,k] T_k(tanh x[b,i])          (paper Eq. 2-3, Alg. 1 inner loop)
// block = (64 outputs, 4 rows); grid = (ceil(B/4), ceil(O/64)).
__global__ void __launch_bounds__(256)
generic_forward_kernel(const float* __restrict__ x, const float* __restrict__ C, float* __restrict__ y,
                       int64_t B, int I, int O, int degree)
{
    const int o = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (o >= O || b >= B) return;
    const int K = degree + 1;
    const float* xr = x + b * I;
    float total = 0.0f, part = 0.0f;
    for (int i = 0; i < I; ++i) {
        float t, w;                              // T_k(|u|), 1 - |u|
        normalise_split(xr[i], t, w);
        const bool neg = xr[i] < 0.0f;
        const float m2w = -2.0f * w;
        const float* c = C + ((int64_t)i * O + o) * K;
        float d = -w;
        float acc = c[0];
        for (int k = 1; k < K; ++k) {
            acc = fmaf(c[k], ((k & 1) && neg) ? -t : t, acc);
            d = fmaf(m2w, t, d);
            t += d;
        }
        part += acc;
        if ((i % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    y[b * O + o] = total + part;
}

// dx[b,i] = (1-u^2) sum_o dy[b,o] sum_{k>=1} C[i,o,k] T_k'(u)   (paper Alg. 2, x_grad)
// block = (64 inputs, 4 rows); grid = (ceil(B/4), ceil(I/64)).
__global__ void __launch_bounds__(256)
generic_dx_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                  float* __restrict__ dx, int64_t B, int I, int O, int degree)
{
    const int i = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (i >= I || b >= B) return;
    const int K = degree + 1;
    float slope;
    const float u = normalise(x[b * I + i], slope);
    const float two_u = 2.0f * u;
    const float* g = dy + b * O;
    float total = 0.0f, part = 0.0f;
    for (int o = 0; o < O; ++o) {
        const float* c = C + ((int64_t)i * O + o) * K;
        float U_prev = 0.0f, U_cur = 1.0f;   // U_{k-2}, U_{k-1}
        float inner = 0.0f;
        for (int k = 1; k < K; ++k) {
            inner = fmaf(c[k], (float)k * U_cur, inner);
            const float U_next = fmaf(two_u, U_cur, -U_prev);
            U_prev = U_cur;
            U_cur = U_next;
        }
        part = fmaf(g[o], inner, part);
        if ((o % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    dx[b * I + i] = slope * (total + part);
}

// dC[i,o,k] = sum_b T_k(tanh x[b,i]) dy[b,o]                   (paper Alg. 2, coeff_grad)
// one thread per coefficient, sequential over the batch in a fixed order.
__global__ void __launch_bounds__(256)
generic_dC_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ dC,
                  int64_t B, int I, int O, int degree)
{
    const int K = degree + 1;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)I * O * K) return;
    const int k = (int)(e % K);
    const int o = (int)((e / K) % O);
    const int i = (int)(e / ((int64_t)K * O));
    float total = 0.0f, mid = 0.0f, part = 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        const float xv = x[b * I + i];
        float t, w;
        normalise_split(xv, t, w);
        const float m2w = -2.0f * w;
        float d = -w;
        for (int n = 1; n < k; ++n) {
            d = fmaf(m2w, t, d);
            t += d;
        }
        const float t_k = (k == 0) ? 1.0f : (((k & 1) && xv < 0.0f) ? -t : t);
        part = fmaf(t_k, dy[b * O + o], part);
        if ((b % 64) == 63) { mid += part; part = 0.0f; }
        if ((b % 4096) == 4095) { total += mid; mid = 0.0f; }
    }
    dC[e] = total + (mid + part);
}

// ------------------------------------------------------------------------------------------
// Table-interpolated variant (paper Sec. 4.2) for any degree and any table size: the table
// LUT[k][i] stays in global memory (it is read through the caches), one thread per output
// element as above.  cell index c = min(floor((u+1)/2 (n-1)), n-2), fraction f = pos - c.
__device__ __forceinline__ int table_cell(float u, int n, float& f)
{
    const float half = 0.5f * (float)(n - 1);
    const float pos = fmaf(u, half, half);
    int c = (int)pos;
    c = c < n - 2 ? c : n - 2;
    f = pos - (float)c;
    return c;
}

__global__ void __launch_bounds__(256)
generic_forward_table_kernel(const float* __restrict__ x, const float* __restrict__ C,
                             const float* __restrict__ lut, int n, float* __restrict__ y, int64_t B, int I, int O,
                             int degree)
{
    const int o = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (o >= O || b >= B) return;
    const int K = degree + 1;
    const float* xr = x + b * I;
    float total = 0.0f, part = 0.0f;
    for (int i = 0; i < I; ++i) {
        float f;
        const int c = table_cell(normalise(xr[i]), n, f);
        const float* cf = C + ((int64_t)i * O + o) * K;
        float acc = 0.0f;
        for (int k = 0; k < K; ++k) {
            const float lo = lut[(int64_t)k * n + c], hi = lut[(int64_t)k * n + c + 1];
            acc = fmaf(cf[k], fmaf(f, hi - lo, lo), acc);
        }
        part += acc;
        if ((i % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    y[b * O + o] = total + part;
}

__global__ void __launch_bounds__(256)
generic_dx_table_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                        const float* __restrict__ lut, int n, float* __restrict__ dx, int64_t B, int I, int O,
                        int degree)
{
    const int i = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (i >= I || b >= B) return;
    const int K = degree + 1;
    float slope, f;
    const int c = table_cell(normalise(x[b * I + i], slope), n, f);
    const float inv_delta = 0.5f * (float)(n - 1);
    const float* g = dy + b * O;
    float total = 0.0f, part = 0.0f;
    for (int o = 0; o < O; ++o) {
        const float* cf = C + ((int64_t)i * O + o) * K;
        float inner = 0.0f;
        for (int k = 1; k < K; ++k)
            inner = fmaf(cf[k], (lut[(int64_t)k * n + c + 1] - lut[(int64_t)k * n + c]) * inv_delta, inner);
        part = fmaf(g[o], inner, part);
        if ((o % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    dx[b * I + i] = slope * (total + part);
}

// dx with the derivative read from the auxiliary table dlut[k][i] = T_k'(-1 + i*Delta), interpolated
// like the values (the second option of Sec. 4.2.2).
__global__ void __launch_bounds__(256)
generic_dx_table2_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                         const float* __restrict__ dlut, int n, float* __restrict__ dx, int64_t B, int I, int O,
                         int degree)
{
    const int i = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (i >= I || b >= B) return;
    const int K = degree + 1;
    float slope, f;
    const int c = table_cell(normalise(x[b * I + i], slope), n, f);
    const float* g = dy + b * O;
    float total = 0.0f, part = 0.0f;
    for (int o = 0; o < O; ++o) {
        const float* cf = C + ((int64_t)i * O + o) * K;
        float inner = 0.0f;
        for (int k = 1; k < K; ++k) {
            const float lo = dlut[(int64_t)k * n + c];
            inner = fmaf(cf[k], fmaf(f, dlut[(int64_t)k * n + c + 1] - lo, lo), inner);
        }
        part = fmaf(g[o], inner, part);
        if ((o % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    dx[b * I + i] = slope * (total + part);
}

__global__ void __launch_bounds__(256)
generic_dC_table_kernel(const float* __restrict__ x, const float* __restrict__ dy, const float* __restrict__ lut,
                        int n, float* __restrict__ dC, int64_t B, int I, int O, int degree)
{
    const int K = degree + 1;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)I * O * K) return;
    const int k = (int)(e % K);
    const int o = (int)((e / K) % O);
    const int i = (int)(e / ((int64_t)K * O));
    const float* row = lut + (int64_t)k * n;
    float total = 0.0f, mid = 0.0f, part = 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        float f;
        const int c = table_cell(normalise(x[b * I + i]), n, f);
        const float lo = row[c];
        part = fmaf(fmaf(f, row[c + 1] - lo, lo), dy[b * O + o], part);
        if ((b % 64) == 63) { mid += part; part = 0.0f; }
        if ((b % 4096) == 4095) { total += mid; mid = 0.0f; }
    }
    dC[e] = total + (mid + part);
}

// ------------------------------------------------------------------------------------------
// Other bases (kind 1 Legendre, 2 Hermite, 3 Fourier; see the policies in basis.h) at any
// degree up to 32: one thread per output element, the basis of one input evaluated into a
// small per-thread array.  bv[k] = B_k, db[k] = dB_k/du (dB_k/dx for Fourier), slope = du/dx.
__device__ inline void family_eval(int kind, float x, int d, float* bv, float* db, float& slope)
{
    bv[0] = 1.0f;
    db[0] = 0.0f;
    if (kind == 3) {
        slope = 1.0f;
        const float c1 = cosf(x), s1 = sinf(x);
        float c = c1, s = s1;
        for (int m = 1; m <= d / 2; ++m) {
            bv[2 * m - 1] = c;
            bv[2 * m] = s;
            db[2 * m - 1] = -(float)m * s;
            db[2 * m] = (float)m * c;
            const float cn = fmaf(c, c1, -s * s1), sn = fmaf(s, c1, c * s1);
            c = cn;
            s = sn;
        }
        return;
    }
    const float u = normalise(x, slope);
    if (d >= 1) {
        bv[1] = kind == 2 ? 2.0f * u : u;
        db[1] = kind == 2 ? 2.0f : 1.0f;
    }
    for (int k = 1; k < d; ++k) {
        if (kind == 2) {
            bv[k + 1] = fmaf(2.0f * u, bv[k], -(float)(2 * k) * bv[k - 1]);
            db[k + 1] = (float)(2 * k + 2) * bv[k];
        } else {
            bv[k + 1] = ((float)(2 * k + 1) * u * bv[k] - (float)k * bv[k - 1]) / (float)(k + 1);
            db[k + 1] = fmaf((float)(2 * k + 1), bv[k], db[k - 1]);
        }
    }
}

constexpr int FAMILY_MAX_K = 33;

__global__ void __launch_bounds__(256)
generic_forward_family_kernel(int kind, const float* __restrict__ x, const float* __restrict__ C,
                              float* __restrict__ y, int64_t B, int I, int O, int degree)
{
    const int o = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (o >= O || b >= B) return;
    const int K = degree + 1;
    float bv[FAMILY_MAX_K], db[FAMILY_MAX_K], slope;
    float total = 0.0f, part = 0.0f;
    for (int i = 0; i < I; ++i) {
        family_eval(kind, x[b * I + i], degree, bv, db, slope);
        const float* cf = C + ((int64_t)i * O + o) * K;
        float acc = 0.0f;
        for (int k = 0; k < K; ++k) acc = fmaf(cf[k], bv[k], acc);
        part += acc;
        if ((i % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    y[b * O + o] = total + part;
}

__global__ void __launch_bounds__(256)
generic_dx_family_kernel(int kind, const float* __restrict__ x, const float* __restrict__ C,
                         const float* __restrict__ dy, float* __restrict__ dx, int64_t B, int I, int O, int degree)
{
    const int i = blockIdx.y * 64 + threadIdx.x;
    const int64_t b = (int64_t)blockIdx.x * 4 + threadIdx.y;
    if (i >= I || b >= B) return;
    const int K = degree + 1;
    float bv[FAMILY_MAX_K], db[FAMILY_MAX_K], slope;
    family_eval(kind, x[b * I + i], degree, bv, db, slope);
    const float* g = dy + b * O;
    float total = 0.0f, part = 0.0f;
    for (int o = 0; o < O; ++o) {
        const float* cf = C + ((int64_t)i * O + o) * K;
        float inner = 0.0f;
        for (int k = 1; k < K; ++k) inner = fmaf(cf[k], db[k], inner);
        part = fmaf(g[o], inner, part);
        if ((o % GENERIC_FOLD) == GENERIC_FOLD - 1) { total += part; part = 0.0f; }
    }
    dx[b * I + i] = slope * (total + part);
}

__global__ void __launch_bounds__(256)
generic_dC_family_kernel(int kind, const float* __restrict__ x, const float* __restrict__ dy,
                         float* __restrict__ dC, int64_t B, int I, int O, int degree)
{
    const int K = degree + 1;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)I * O * K) return;
    const int k = (int)(e % K);
    const int o = (int)((e / K) % O);
    const int i = (int)(e / ((int64_t)K * O));
    float bv[FAMILY_MAX_K], db[FAMILY_MAX_K], slope;
    float total = 0.0f, mid = 0.0f, part = 0.0f;
    for (int64_t b = 0; b < B; ++b) {
        family_eval(kind, x[b * I + i], degree, bv, db, slope);
        part = fmaf(bv[k], dy[b * O + o], part);
        if ((b % 64) == 63) { mid += part; part = 0.0f; }
        if ((b % 4096) == 4095) { total += mid; mid = 0.0f; }
    }
    dC[e] = total + (mid + part);
}

}  // namespace chebykan
