// Device-side Chebyshev basis helpers shared by every kernel of the library.
//
// u = tanh(x) maps the input into [-1,1] (paper Sec. 4.2, Fig. 3 caption);
// T_k follows the three-term recurrence of Eq. 2; the derivative uses
// T_k' = k U_{k-1} with the second-kind recurrence, which stays finite at
// u = +-1 (the trigonometric derivative form does not).
#pragma once
#include <hip/hip_runtime.h>

namespace chebykan {

__device__ __forceinline__ float normalise(float x) { return tanhf(x); }

// 1 - u^2 without cancellation for |u| close to 1: (1-u) is exact there.
__device__ __forceinline__ float tanh_slope(float u) { return (1.0f - u) * (1.0f + u); }

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

}  // namespace chebykan
