// Device-side Chebyshev basis helpers shared by every kernel of the library.
//
// u = tanh(x) maps the input into [-1,1] (paper Sec. 4.2, Fig. 3 caption);
// T_k follows the three-term recurrence of Eq. 2; the derivative uses
// T_k' = k U_{k-1} with the second-kind recurrence, which stays finite at
// u = +-1 (the trigonometric derivative form does not).
#pragma once
#include <hip/hip_runtime.h>

namespace chebykan {

// u = tanh(x) = 1 - 2t/(1+t) with t = exp(-2|x|), on the hardware exp2 and reciprocal
// units (about 1 ulp each).  In this form the absolute error is smallest where |u| -> 1,
// which is where T_k' (up to k^2) amplifies it; over x ~ N(0,1) the resulting basis error
// is within 30 % of what a correctly rounded tanh gives (u: rms 5e-8, max 2.5e-7 absolute;
// relative accuracy of u itself is lost for |x| < 1e-3, which no output is sensitive to).
// |x| > 44 gives t = 0 and u = +-1 exactly; NaN propagates.
__device__ __forceinline__ float normalise(float x)
{
    const float ax = fabsf(x);
    const float t2 = __builtin_amdgcn_exp2f(fmaf(ax, -2.885390081777927f, 1.0f));   // 2 exp(-2|x|)
    const float r = __builtin_amdgcn_rcpf(fmaf(0.5f, t2, 1.0f));                      // 1 / (1 + t)
    return copysignf(fmaf(-t2, r, 1.0f), x);
}

// Same u, plus the tanh derivative 1 - u^2 = 4t/(1+t)^2 taken from t directly, which keeps
// its relative accuracy in the tails where 1 - u*u would cancel.
__device__ __forceinline__ float normalise(float x, float& slope)
{
    const float ax = fabsf(x);
    const float t2 = __builtin_amdgcn_exp2f(fmaf(ax, -2.885390081777927f, 1.0f));
    const float r = __builtin_amdgcn_rcpf(fmaf(0.5f, t2, 1.0f));
    slope = (t2 * r) * (r + r);
    return copysignf(fmaf(-t2, r, 1.0f), x);
}

// |u| and w = 1 - |u| = 2t/(1+t) from the same t; w keeps full relative accuracy as |u| -> 1.
__device__ __forceinline__ void normalise_split(float x, float& abs_u, float& w)
{
    const float ax = fabsf(x);
    const float t2 = __builtin_amdgcn_exp2f(fmaf(ax, -2.885390081777927f, 1.0f));
    const float r = __builtin_amdgcn_rcpf(fmaf(0.5f, t2, 1.0f));
    w = t2 * r;
    abs_u = fmaf(-t2, r, 1.0f);
}

// T[0..D] at u.
template <int D>
__device__ __forceinline__ void cheb_T(float u, float (&T)[D + 1])
{
    T[0] = 1.0f;
    if constexpr (D >= 1) T[1] = u;
    const float two_u = 2.0f * u;
#pragma unroll
    for (int k = 1; k < D; ++k) T[k + 1] = fmaf(two_u, T[k], -T[k - 1]);
}

// T[0..D] at u = tanh(x), straight from x.  Up to degree 8 this is normalise() + cheb_T().
// Above that the plain recurrence loses accuracy where |u| -> 1 (an absolute error in u is
// amplified by T_k' ~ k^2), so the recurrence is run in difference form on w = 1 - |u|, which
// the tanh yields with full RELATIVE accuracy (w = 2t/(1+t)):
//     d_1 = -w,  d_{k+1} = d_k - 2 w T_k,  T_{k+1} = T_k + d_{k+1}        (T_k at |u|)
// and T_k(u) = sign(x)^k T_k(|u|).  Algebraically identical to Eq. 2.
template <int D>
__device__ __forceinline__ void cheb_T_of_x(float x, float (&T)[D + 1])
{
    if constexpr (D <= 8) {
        cheb_T<D>(normalise(x), T);
    } else {
        float Tk, w;                                     // |u|, 1 - |u|
        normalise_split(x, Tk, w);
        const float m2w = -2.0f * w;
        float d = -w;
        T[0] = 1.0f;
        T[1] = copysignf(Tk, x);
#pragma unroll
        for (int k = 1; k < D; ++k) {
            d = fmaf(m2w, Tk, d);
            Tk += d;
            T[k + 1] = ((k + 1) & 1) ? (x < 0.0f ? -Tk : Tk) : Tk;
        }
    }
}

// dT[k-1] = T_k'(u) for k = 1..D   (T_0' = 0 is not stored).
template <int D>
__device__ __forceinline__ void cheb_dT(float u, float (&dT)[D > 0 ? D : 1])
{
    if constexpr (D >= 1) {
        const float two_u = 2.0f * u;
        float U_prev = 0.0f, U_cur = 1.0f;
#pragma unroll
        for (int k = 1; k <= D; ++k) {
            dT[k - 1] = (float)k * U_cur;
            const float U_next = fmaf(two_u, U_cur, -U_prev);
            U_prev = U_cur;
            U_cur = U_next;
        }
    }
}

// ---------------------------------------------------------------- basis policies
// A kernel obtains T_k and T_k' through one of two policies with the same interface.
//
// ExactBasis: the recurrences above (the default path).
//
// TableBasis: the paper's lookup-table variant (Sec. 4.2).  The caller's table
// LUT[k][i] = T_k(-1 + i*Delta), Delta = 2/(n-1), is staged once per workgroup into LDS,
// transposed to [i][K] so that the 2K values of a cell are adjacent.  Online (Sec. 4.2.2):
// pos = (u+1)/2 (n-1), c = min(floor(pos), n-2), f = pos - c,
//     T_k  ~ LUT[k][c] + f (LUT[k][c+1] - LUT[k][c])
//     T_k' ~ (LUT[k][c+1] - LUT[k][c]) / Delta          (difference of neighbouring samples)
// The paper keeps its table in global memory because it does not fit the on-chip memory of
// its GPU; 160 KB of LDS per compute unit hold tables of a few thousand samples.
struct ExactBasis {
    static constexpr bool kTable = false;
    static constexpr int kTableRows = 0;   // tables staged per sample: 0 none, 1 values, 2 values and derivatives
    struct Args {};
    __device__ ExactBasis(const Args&, float*, int, int, int) {}
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        cheb_T_of_x<D>(x, out);
    }
    // dT[k-1] = T_k', slope = 1 - tanh(x)^2
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        const float u = normalise(x, slope);
        cheb_dT<D>(u, out);
    }
    // both at once; the derivative only where `want_dt` holds
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool want_dt) const
    {
        const float u = normalise(x, slope);
        if constexpr (D <= 8) cheb_T<D>(u, t);
        else cheb_T_of_x<D>(x, t);
        if (want_dt) cheb_dT<D>(u, dt);
    }
};

// Other KAN bases on the same skeleton (paper Sec. 2.3: alpha_k B_{k+1} = beta_k(x) B_k - gamma_k B_{k-1};
// Sec. 6.3 reports the method on Fourier, Legendre and Hermite KANs).  The paper prints no
// formulas for them; the textbook recurrences are used.  In every family B_0 = 1, so the input
// gradient skips k = 0 exactly as for Chebyshev.  `slope` is the factor the kernels multiply the
// k-sum with: 1 - tanh(x)^2 for the polynomial families (dT is then dB_k/du), 1 for Fourier
// (dT is dB_k/dx).
struct LegendreBasis {   // (k+1) P_{k+1} = (2k+1) u P_k - k P_{k-1};  P'_{k+1} = P'_{k-1} + (2k+1) P_k;  u = tanh x
    static constexpr bool kTable = false;
    static constexpr int kTableRows = 0;
    struct Args {};
    __device__ LegendreBasis(const Args&, float*, int, int, int) {}
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        const float u = normalise(x);
        out[0] = 1.0f;
        if constexpr (D >= 1) out[1] = u;
#pragma unroll
        for (int k = 1; k < D; ++k)
            out[k + 1] = fmaf((float)(2 * k + 1) / (float)(k + 1) * u, out[k], -(float)k / (float)(k + 1) * out[k - 1]);
    }
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool) const
    {
        const float u = normalise(x, slope);
        t[0] = 1.0f;
        if constexpr (D >= 1) { t[1] = u; dt[0] = 1.0f; }
#pragma unroll
        for (int k = 1; k < D; ++k) {
            t[k + 1] = fmaf((float)(2 * k + 1) / (float)(k + 1) * u, t[k], -(float)k / (float)(k + 1) * t[k - 1]);
            dt[k] = fmaf((float)(2 * k + 1), t[k], k >= 2 ? dt[k - 2] : 0.0f);   // P'_{k+1}; P'_0 = 0
        }
    }
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        float t[D + 1];
        T_dT<D>(x, t, out, slope, true);
    }
};

struct HermiteBasis {    // physicists': H_{k+1} = 2 u H_k - 2k H_{k-1};  H'_k = 2k H_{k-1};  u = tanh x
    static constexpr bool kTable = false;
    static constexpr int kTableRows = 0;
    struct Args {};
    __device__ HermiteBasis(const Args&, float*, int, int, int) {}
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        const float two_u = 2.0f * normalise(x);
        out[0] = 1.0f;
        if constexpr (D >= 1) out[1] = two_u;
#pragma unroll
        for (int k = 1; k < D; ++k) out[k + 1] = fmaf(two_u, out[k], -(float)(2 * k) * out[k - 1]);
    }
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool) const
    {
        const float two_u = 2.0f * normalise(x, slope);
        t[0] = 1.0f;
        if constexpr (D >= 1) t[1] = two_u;
#pragma unroll
        for (int k = 1; k < D; ++k) t[k + 1] = fmaf(two_u, t[k], -(float)(2 * k) * t[k - 1]);
#pragma unroll
        for (int k = 1; k <= D; ++k) dt[k - 1] = (float)(2 * k) * t[k - 1];
    }
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        float t[D + 1];
        T_dT<D>(x, t, out, slope, true);
    }
};

struct FourierBasis {    // B_0 = 1, B_{2m-1} = cos(m x), B_{2m} = sin(m x) on the raw input; D = 2G
    static constexpr bool kTable = false;
    static constexpr int kTableRows = 0;
    struct Args {};
    __device__ FourierBasis(const Args&, float*, int, int, int) {}
    // cos(m x), sin(m x) for m = 1..G from cos x, sin x by the angle-addition recurrence (Sec. 2.3)
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        static_assert(D % 2 == 0, "Fourier basis: the degree counts cos/sin pairs");
        const float c1 = cosf(x), s1 = sinf(x);
        float c = c1, s = s1;
        out[0] = 1.0f;
#pragma unroll
        for (int m = 1; m <= D / 2; ++m) {
            out[2 * m - 1] = c;
            out[2 * m] = s;
            const float cn = fmaf(c, c1, -s * s1), sn = fmaf(s, c1, c * s1);
            c = cn;
            s = sn;
        }
    }
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool) const
    {
        T<D>(x, t);
        slope = 1.0f;
#pragma unroll
        for (int m = 1; m <= D / 2; ++m) {
            dt[2 * m - 2] = -(float)m * t[2 * m];       // d cos(m x)/dx
            dt[2 * m - 1] = (float)m * t[2 * m - 1];    // d sin(m x)/dx
        }
    }
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        float t[D + 1];
        T_dT<D>(x, t, out, slope, true);
    }
};

struct TableBasis {
    static constexpr bool kTable = true;
    static constexpr int kTableRows = 1;
    struct Args {
        const float* lut;   // device, [K][n]
        int n;              // samples per row
    };
    const float* tab;       // LDS, [n][K]
    float half;             // (n-1)/2
    float inv_delta;        // (n-1)/2
    int last;               // n-2

    // Stage the table into LDS at `dst` (n*K floats).  Every thread of the workgroup calls this;
    // it ends with a barrier.
    __device__ TableBasis(const Args& a, float* dst, int K, int tid, int nthreads)
    {
        const int total = a.n * K;
        for (int e = tid; e < total; e += nthreads) {
            const int k = e / a.n, i = e - k * a.n;
            dst[i * K + k] = a.lut[e];
        }
        __syncthreads();
        tab = dst;
        half = 0.5f * (float)(a.n - 1);
        inv_delta = half;
        last = a.n - 2;
    }

    // cell base pointer and in-cell fraction for u in [-1, 1]
    template <int K>
    __device__ __forceinline__ const float* cell(float u, float& frac) const
    {
        const float pos = fmaf(u, half, half);
        int c = (int)pos;                       // pos >= 0: truncation is the floor
        c = c < last ? c : last;
        frac = pos - (float)c;
        return tab + c * K;
    }
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        float f;
        const float* p = cell<D + 1>(normalise(x), f);
#pragma unroll
        for (int k = 0; k <= D; ++k) out[k] = fmaf(f, p[D + 1 + k] - p[k], p[k]);
    }
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        float f;
        const float* p = cell<D + 1>(normalise(x, slope), f);
#pragma unroll
        for (int k = 1; k <= D; ++k) out[k - 1] = (p[D + 1 + k] - p[k]) * inv_delta;
    }
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool) const
    {
        float f;
        const float* p = cell<D + 1>(normalise(x, slope), f);
#pragma unroll
        for (int k = 0; k <= D; ++k) {
            const float lo = p[k], diff = p[D + 1 + k] - lo;
            t[k] = fmaf(f, diff, lo);
            if (k >= 1) dt[k - 1] = diff * inv_delta;
        }
    }
};

// DerivTableBasis: the table variant whose derivative comes from a second table (the auxiliary-table
// option of Sec. 4.2.2, read as samples dLUT[k][i] = T_k'(-1 + i*Delta) interpolated like the
// values: second order in Delta where the difference quotient of one cell is first order, and
// continuous across knots).  Both tables are staged into LDS interleaved per sample,
// [i][0..K) = T_k, [i][K..2K) = T_k', so that the 4K numbers of a cell are adjacent.
struct DerivTableBasis {
    static constexpr bool kTable = true;
    static constexpr int kTableRows = 2;
    struct Args {
        const float* lut;    // device, [K][n] values
        const float* dlut;   // device, [K][n] derivatives
        int n;               // samples per row
    };
    const float* tab;        // LDS, [n][2K]
    float half;              // (n-1)/2
    int last;                // n-2

    __device__ DerivTableBasis(const Args& a, float* dst, int K, int tid, int nthreads)
    {
        const int total = a.n * K;
        for (int e = tid; e < total; e += nthreads) {
            const int k = e / a.n, i = e - k * a.n;
            dst[i * 2 * K + k] = a.lut[e];
            dst[i * 2 * K + K + k] = a.dlut[e];
        }
        __syncthreads();
        tab = dst;
        half = 0.5f * (float)(a.n - 1);
        last = a.n - 2;
    }
    template <int K>
    __device__ __forceinline__ const float* cell(float u, float& frac) const
    {
        const float pos = fmaf(u, half, half);
        int c = (int)pos;                       // pos >= 0: truncation is the floor
        c = c < last ? c : last;
        frac = pos - (float)c;
        return tab + c * 2 * K;
    }
    template <int D>
    __device__ __forceinline__ void T(float x, float (&out)[D + 1]) const
    {
        constexpr int K = D + 1;
        float f;
        const float* p = cell<K>(normalise(x), f);
#pragma unroll
        for (int k = 0; k < K; ++k) out[k] = fmaf(f, p[2 * K + k] - p[k], p[k]);
    }
    template <int D>
    __device__ __forceinline__ void dT(float x, float (&out)[D > 0 ? D : 1], float& slope) const
    {
        constexpr int K = D + 1;
        float f;
        const float* p = cell<K>(normalise(x, slope), f);
#pragma unroll
        for (int k = 1; k < K; ++k) out[k - 1] = fmaf(f, p[3 * K + k] - p[K + k], p[K + k]);
    }
    template <int D>
    __device__ __forceinline__ void T_dT(float x, float (&t)[D + 1], float (&dt)[D > 0 ? D : 1], float& slope,
                                         bool) const
    {
        constexpr int K = D + 1;
        float f;
        const float* p = cell<K>(normalise(x, slope), f);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            t[k] = fmaf(f, p[2 * K + k] - p[k], p[k]);
            if (k >= 1) dt[k - 1] = fmaf(f, p[3 * K + k] - p[K + k], p[K + k]);
        }
    }
};

}  // namespace chebykan
