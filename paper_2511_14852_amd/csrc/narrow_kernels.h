// Kernels for layers with very few outputs (out <= 4, e.g. a regression head).
//
// With so few outputs the layer is not a matrix product but a stream over x:
// forward is a per-row reduction over the input features, backward is
// elementwise in dx and a column reduction over the batch in dC.  Both are bound
// by HBM traffic (x is read once per pass, dx written once), so they run on the
// vector ALUs with coalesced row-major accesses: consecutive lanes take
// consecutive input features of one row.
//
//   forward   y[b,o]    = sum_i sum_k C[i,o,k] T_k(tanh x[b,i])        (paper Eq. 2-3)
//   backward  dx[b,i]   = (1-u^2) sum_o dy[b,o] sum_{k>=1} C[i,o,k] T_k'(u)
//             dC[i,o,k] = sum_b T_k(u) dy[b,o]                          (paper Alg. 2)
//
// dx and dC come out of ONE pass over x.  dC is reduced without atomics: each
// thread sums its own rows, the row groups of a workgroup are added through LDS
// in a fixed order, and each workgroup writes one partial buffer that a second
// kernel adds in slice order (the two-stage reduction of Sec. 4.4 on the batch
// axis).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "basis.h"

namespace chebykan {

constexpr int NARROW_THREADS = 256;
constexpr int NARROW_RB = 4;   // rows in flight per lane (memory-level parallelism)

// lanes [0,G) of each aligned group of G lanes hold partial sums of one row
__device__ __forceinline__ float group_sum(float v, int G)
{
    for (int m = G >> 1; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// grid.x workgroups, each owning `rows_per_wg` consecutive rows; G = lanes per row
// (power of two, 8..64).  Dynamic LDS: I*O*(D+1) floats, coefficients as [k][o][i].
template <int D, int O>
__global__ void __launch_bounds__(NARROW_THREADS)
narrow_fwd_kernel(const float* __restrict__ x, const float* __restrict__ C, float* __restrict__ y,
                  int B, int I, int G, int rows_per_wg)
{
    constexpr int K = D + 1;
    extern __shared__ __align__(16) float lds[];
    const int t = threadIdx.x;
    for (int e = t; e < I * O * K; e += NARROW_THREADS) {
        const int k = e % K, o = (e / K) % O, i = e / (K * O);
        lds[(k * O + o) * I + i] = C[e];
    }
    __syncthreads();

    const int g = t % G, rg = t / G, RPW = NARROW_THREADS / G;
    const int64_t first = (int64_t)blockIdx.x * rows_per_wg;
    int64_t last = first + rows_per_wg;
    if (last > B) last = B;
    const int nj = (I + G - 1) / G;

    // every thread runs the same number of iterations (the group sums below need whole waves)
    const int n_iter = (rows_per_wg + NARROW_RB * RPW - 1) / (NARROW_RB * RPW);
    for (int it = 0; it < n_iter; ++it) {
        const int64_t row0 = first + rg + (int64_t)it * NARROW_RB * RPW;
        float part[NARROW_RB][O];
#pragma unroll
        for (int r = 0; r < NARROW_RB; ++r)
#pragma unroll
            for (int o = 0; o < O; ++o) part[r][o] = 0.0f;
        for (int j = 0; j < nj; ++j) {
            const int i = g + j * G;
            if (i < I) {
                float xv[NARROW_RB];
#pragma unroll
                for (int r = 0; r < NARROW_RB; ++r) {
                    const int64_t row = row0 + (int64_t)r * RPW;
                    xv[r] = row < last ? x[row * I + i] : 0.0f;
                }
                float cs[O][K];
#pragma unroll
                for (int o = 0; o < O; ++o)
#pragma unroll
                    for (int k = 0; k < K; ++k) cs[o][k] = lds[(k * O + o) * I + i];
#pragma unroll
                for (int r = 0; r < NARROW_RB; ++r) {
                    float T[K];
                    cheb_T<D>(normalise(xv[r]), T);
#pragma unroll
                    for (int o = 0; o < O; ++o) {
                        float s = 0.0f;
#pragma unroll
                        for (int k = 0; k < K; ++k) s = fmaf(cs[o][k], T[k], s);
                        part[r][o] += s;
                    }
                }
            }
        }
#pragma unroll
        for (int r = 0; r < NARROW_RB; ++r) {
            const int64_t row = row0 + (int64_t)r * RPW;
#pragma unroll
            for (int o = 0; o < O; ++o) {
                const float s = group_sum(part[r][o], G);
                if (g == 0 && row < last) y[row * O + o] = s;
            }
        }
    }
}

template <int O> struct NarrowFpl { static constexpr int value = (4 / O) > 0 ? (4 / O) : 1; };

// grid = (row slices, feature blocks of G*FPL features).  Writes dx (if non-null) and
// partial[slice][i][o][k] (if non-null).  Dynamic LDS: 256*FPL*O*(D+1) floats.
template <int D, int O>
__global__ void __launch_bounds__(NARROW_THREADS)
narrow_bwd_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                  float* __restrict__ dx, float* __restrict__ partial, int B, int I, int G, int rows_per_wg)
{
    constexpr int K = D + 1, FPL = NarrowFpl<O>::value;
    extern __shared__ __align__(16) float lds[];
    const int t = threadIdx.x;
    const int g = t % G, rg = t / G, RPW = NARROW_THREADS / G;
    const int i_first = blockIdx.y * G * FPL + g;
    const int64_t first = (int64_t)blockIdx.x * rows_per_wg;
    int64_t last = first + rows_per_wg;
    if (last > B) last = B;

    // feature groups of this block that exist at all (uniform over the workgroup)
    int nj = (I - (int)blockIdx.y * G * FPL + G - 1) / G;
    if (nj > FPL) nj = FPL;

    float creg[FPL][O][D > 0 ? D : 1];   // C[i,o,1..D]: only the input gradient needs coefficients
    float acc[FPL][O][K];
#pragma unroll
    for (int j = 0; j < FPL; ++j) {
        const int i = i_first + j * G;
#pragma unroll
        for (int o = 0; o < O; ++o) {
#pragma unroll
            for (int k = 0; k < K; ++k) acc[j][o][k] = 0.0f;
#pragma unroll
            for (int k = 1; k < K; ++k) creg[j][o][k - 1] = (i < I && dx) ? C[((int64_t)i * O + o) * K + k] : 0.0f;
        }
    }

    const int n_iter = (rows_per_wg + NARROW_RB * RPW - 1) / (NARROW_RB * RPW);
    for (int it = 0; it < n_iter; ++it) {
        const int64_t row0 = first + rg + (int64_t)it * NARROW_RB * RPW;
        float xv[NARROW_RB][FPL];
        float gv[NARROW_RB][O];
#pragma unroll
        for (int r = 0; r < NARROW_RB; ++r) {
            const int64_t row = row0 + (int64_t)r * RPW;
            const bool ok = row < last;
#pragma unroll
            for (int o = 0; o < O; ++o) gv[r][o] = ok ? dy[row * O + o] : 0.0f;   // zero rows add nothing
#pragma unroll
            for (int j = 0; j < FPL; ++j) {
                const int i = i_first + j * G;
                xv[r][j] = (j < nj && ok && i < I) ? x[row * I + i] : 0.0f;
            }
        }
#pragma unroll
        for (int r = 0; r < NARROW_RB; ++r) {
            const int64_t row = row0 + (int64_t)r * RPW;
#pragma unroll
            for (int j = 0; j < FPL; ++j) {
                if (j >= nj) continue;
                const int i = i_first + j * G;
                float slope;
                const float u = normalise(xv[r][j], slope);
                float T[K];
                cheb_T<D>(u, T);
#pragma unroll
                for (int o = 0; o < O; ++o)
#pragma unroll
                    for (int k = 0; k < K; ++k) acc[j][o][k] = fmaf(T[k], gv[r][o], acc[j][o][k]);
                if constexpr (D >= 1) {
                    if (dx && row < last && i < I) {
                        float dT[D];
                        cheb_dT<D>(u, dT);
                        float s = 0.0f;
#pragma unroll
                        for (int o = 0; o < O; ++o) {
                            float inner = 0.0f;
#pragma unroll
                            for (int k = 0; k < D; ++k) inner = fmaf(creg[j][o][k], dT[k], inner);
                            s = fmaf(gv[r][o], inner, s);
                        }
                        dx[row * I + i] = slope * s;
                    }
                }
            }
        }
    }

    if (partial) {
        // row groups of this workgroup, added in index order
        constexpr int PER = FPL * O * K;
#pragma unroll
        for (int j = 0; j < FPL; ++j)
#pragma unroll
            for (int o = 0; o < O; ++o)
#pragma unroll
                for (int k = 0; k < K; ++k) lds[(rg * PER + (j * O + o) * K + k) * G + g] = acc[j][o][k];
        __syncthreads();
        if (rg == 0) {
            float* out = partial + (int64_t)blockIdx.x * I * O * K;
#pragma unroll
            for (int j = 0; j < FPL; ++j) {
                const int i = i_first + j * G;
#pragma unroll
                for (int o = 0; o < O; ++o)
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        float s = 0.0f;
                        for (int q = 0; q < RPW; ++q) s += lds[(q * PER + (j * O + o) * K + k) * G + g];
                        if (i < I) out[((int64_t)i * O + o) * K + k] = s;
                    }
            }
        }
    }
}

// out[e] = sum_s partial[s][e], slices added in a fixed order: 32 slice groups take
// every 32nd slice each, then the 32 group sums are added in group order.
// block = 256 threads = 32 slice groups x 8 elements; grid.x = ceil(n/8).
// Dynamic LDS: 32 x 9 floats.
__global__ void __launch_bounds__(256)
sum_slices_kernel(const float* __restrict__ partial, float* __restrict__ out, int n, int n_slices)
{
    extern __shared__ __align__(16) float lds[];
    const int el = threadIdx.x & 7, sg = threadIdx.x >> 3;
    const int e = blockIdx.x * 8 + el;
    float s = 0.0f;
    if (e < n)
        for (int q = sg; q < n_slices; q += 32) s += partial[(int64_t)q * n + e];
    lds[sg * 9 + el] = s;
    __syncthreads();
    if (sg == 0 && e < n) {
        float total = 0.0f;
#pragma unroll
        for (int q = 0; q < 32; ++q) total += lds[q * 9 + el];
        out[e] = total;
    }
}

}  // namespace chebykan
