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
#include "plans.h"

namespace chebykan {


// Sum over each aligned group of G lanes (G = 8, 16, 32 or 64) with data-parallel-primitive
// adds: shifts inside a row of 16 lanes, then the two row broadcasts of wave64.  The sum of
// a group ends up in its LAST lane; other lanes hold partial sums.  Out-of-row sources read
// as zero (bound_ctrl).
__device__ __forceinline__ float dpp_add(float v, float src, int ctrl_row_mask_sel)
{
    // ctrl_row_mask_sel selects one of the fixed (dpp_ctrl, row_mask) pairs below: the builtin
    // needs compile-time constants
    int r;
    const int x = __builtin_bit_cast(int, src);
    switch (ctrl_row_mask_sel) {
        case 0: r = __builtin_amdgcn_update_dpp(0, x, 0x111, 0xf, 0xf, true); break;   // row_shr:1
        case 1: r = __builtin_amdgcn_update_dpp(0, x, 0x112, 0xf, 0xf, true); break;   // row_shr:2
        case 2: r = __builtin_amdgcn_update_dpp(0, x, 0x114, 0xf, 0xf, true); break;   // row_shr:4
        case 3: r = __builtin_amdgcn_update_dpp(0, x, 0x118, 0xf, 0xf, true); break;   // row_shr:8
        case 4: r = __builtin_amdgcn_update_dpp(0, x, 0x142, 0xa, 0xf, true); break;   // row_bcast:15 -> rows 1,3
        default: r = __builtin_amdgcn_update_dpp(0, x, 0x143, 0xc, 0xf, true); break;  // row_bcast:31 -> rows 2,3
    }
    return v + __builtin_bit_cast(float, r);
}

__device__ __forceinline__ float group_sum(float v, int G)
{
    v = dpp_add(v, v, 0);
    v = dpp_add(v, v, 1);
    v = dpp_add(v, v, 2);
    if (G >= 16) v = dpp_add(v, v, 3);
    if (G >= 32) v = dpp_add(v, v, 4);
    if (G >= 64) v = dpp_add(v, v, 5);
    return v;
}

// Row layout shared by both kernels: a workgroup owns `rows_per_wg` consecutive rows
// (a multiple of NARROW_RB * 256/G); lane group rg of step `it` takes the NARROW_RB
// consecutive rows starting at first + (it * 256/G + rg) * NARROW_RB.  G = lanes per row
// (power of two, 8..64); lane g of a group takes input features g, g+G, ...

// LDS floats of the two kernels' own data (a basis table, if any, follows them)
__host__ __device__ constexpr size_t narrow_fwd_lds_floats(int I, int O, int K) { return ((size_t)I * O * K + 3) & ~(size_t)3; }
__host__ __device__ constexpr size_t narrow_bwd_lds_floats(int O, int K) { return (size_t)NARROW_THREADS * O * K; }

// Both kernels work on a window of O columns of a wider layer: the layer has o_stride outputs
// (row stride of y and dy, output stride of C) and the window starts at column o_begin.  A narrow
// layer is its own window (o_stride = O, o_begin = 0); the 1..4 columns a wide layer has beyond a
// multiple of 128 are a window at its right edge.

// grid.x workgroups.  Dynamic LDS: I*O*(D+1) floats, coefficients as [k][o][i].
// The x values of the next step are requested before the current step is computed.
template <int D, int O, class Basis = ExactBasis>
__global__ void __launch_bounds__(NARROW_THREADS)
narrow_fwd_kernel(const float* __restrict__ x, const float* __restrict__ C, float* __restrict__ y,
                  int B, int I, int G, int rows_per_wg, typename Basis::Args bargs, int o_stride, int o_begin)
{
    constexpr int K = D + 1, RB = NARROW_RB;
    extern __shared__ __align__(16) float lds[];
    const int t = threadIdx.x;
    const Basis basis(bargs, lds + narrow_fwd_lds_floats(I, O, K), K, t, NARROW_THREADS);
    const int g = t % G, rg = t / G, RPW = NARROW_THREADS / G;
    const int64_t first = (int64_t)blockIdx.x * rows_per_wg;
    int64_t last = first + rows_per_wg;
    if (last > B) last = B;
    const int nj = (I + G - 1) / G;
    // every thread runs the same number of steps (the group sums need whole waves)
    const int n_iter = rows_per_wg / (RB * RPW);
    const int n_items = n_iter * nj;

    auto load_item = [&](int w, float (&xv)[RB]) {
        const int it = w / nj, j = w % nj;
        const int i = g + j * G;
        const int64_t row0 = first + ((int64_t)it * RPW + rg) * RB;
#pragma unroll
        for (int r = 0; r < RB; ++r) xv[r] = (i < I && row0 + r < last) ? x[(row0 + r) * I + i] : 0.0f;
    };

    float xnext[RB];
    load_item(0, xnext);
    // consecutive threads fill consecutive LDS words (no bank conflicts); the strided gather from C is tiny
    for (int f = t; f < I * O * K; f += NARROW_THREADS) {
        const int i = f % I, ko = f / I;
        lds[f] = C[((int64_t)i * o_stride + o_begin + ko % O) * K + ko / O];
    }
    __syncthreads();

    float part[RB][O];
    for (int w = 0; w < n_items; ++w) {
        float xv[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) xv[r] = xnext[r];
        if (w + 1 < n_items) load_item(w + 1, xnext);
        const int it = w / nj, j = w % nj;
        const int i = g + j * G;
        if (j == 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int o = 0; o < O; ++o) part[r][o] = 0.0f;
        }
        if (i < I) {
            float cs[O][K];
#pragma unroll
            for (int o = 0; o < O; ++o)
#pragma unroll
                for (int k = 0; k < K; ++k) cs[o][k] = lds[(k * O + o) * I + i];
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                float T[K];
                basis.template T<D>(xv[r], T);
#pragma unroll
                for (int o = 0; o < O; ++o) {
                    float s = 0.0f;
#pragma unroll
                    for (int k = 0; k < K; ++k) s = fmaf(cs[o][k], T[k], s);
                    part[r][o] += s;
                }
            }
        }
        if (j == nj - 1) {
            const int64_t row0 = first + ((int64_t)it * RPW + rg) * RB;
#pragma unroll
            for (int r = 0; r < RB; ++r)
#pragma unroll
                for (int o = 0; o < O; ++o) {
                    const float s = group_sum(part[r][o], G);
                    if (g == G - 1 && row0 + r < last) y[(row0 + r) * o_stride + o_begin + o] = s;
                }
        }
    }
}

// grid = (row slices, ceil(I/G) feature groups).  Writes dx (if non-null) and
// partial[slice][i][o][k] (if non-null).  Dynamic LDS: 256*O*(D+1) floats.
template <int D, int O, class Basis = ExactBasis>
__global__ void __launch_bounds__(NARROW_THREADS)
narrow_bwd_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                  float* __restrict__ dx, float* __restrict__ partial, int B, int I, int G, int rows_per_wg,
                  typename Basis::Args bargs, int o_stride, int o_begin)
{
    constexpr int K = D + 1, RB = NARROW_RB;
    extern __shared__ __align__(16) float lds[];
    const int t = threadIdx.x;
    const Basis basis(bargs, lds + narrow_bwd_lds_floats(O, K), K, t, NARROW_THREADS);
    const int g = t % G, rg = t / G, RPW = NARROW_THREADS / G;
    const int i = blockIdx.y * G + g;
    const bool i_ok = i < I;
    const int64_t first = (int64_t)blockIdx.x * rows_per_wg;
    int64_t last = first + rows_per_wg;
    if (last > B) last = B;
    const int n_iter = rows_per_wg / (RB * RPW);

    auto load_item = [&](int it, float (&xv)[RB], float (&gv)[RB][O]) {
        const int64_t row0 = first + ((int64_t)it * RPW + rg) * RB;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const bool ok = row0 + r < last;
            xv[r] = (ok && i_ok) ? x[(row0 + r) * I + i] : 0.0f;
#pragma unroll
            for (int o = 0; o < O; ++o) gv[r][o] = ok ? dy[(row0 + r) * o_stride + o_begin + o] : 0.0f;   // zero rows add nothing
        }
    };

    float xnext[RB], gnext[RB][O];
    load_item(0, xnext, gnext);

    float creg[O][D > 0 ? D : 1];   // C[i,o,1..D]: only the input gradient needs coefficients
    float acc[O][K];
#pragma unroll
    for (int o = 0; o < O; ++o) {
#pragma unroll
        for (int k = 0; k < K; ++k) acc[o][k] = 0.0f;
#pragma unroll
        for (int k = 1; k < K; ++k) creg[o][k - 1] = (i_ok && dx) ? C[((int64_t)i * o_stride + o_begin + o) * K + k] : 0.0f;
    }

    for (int it = 0; it < n_iter; ++it) {
        float xv[RB], gv[RB][O];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            xv[r] = xnext[r];
#pragma unroll
            for (int o = 0; o < O; ++o) gv[r][o] = gnext[r][o];
        }
        if (it + 1 < n_iter) load_item(it + 1, xnext, gnext);
        const int64_t row0 = first + ((int64_t)it * RPW + rg) * RB;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            float slope;
            float T[K];
            float dT[D > 0 ? D : 1];
            const bool want_dx = dx && i_ok && row0 + r < last;
            basis.template T_dT<D>(xv[r], T, dT, slope, want_dx);
#pragma unroll
            for (int o = 0; o < O; ++o)
#pragma unroll
                for (int k = 0; k < K; ++k) acc[o][k] = fmaf(T[k], gv[r][o], acc[o][k]);
            if constexpr (D >= 1) {
                if (want_dx) {
                    float s = 0.0f;
#pragma unroll
                    for (int o = 0; o < O; ++o) {
                        float inner = 0.0f;
#pragma unroll
                        for (int k = 0; k < D; ++k) inner = fmaf(creg[o][k], dT[k], inner);
                        s = fmaf(gv[r][o], inner, s);
                    }
                    dx[(row0 + r) * I + i] = slope * s;
                }
            }
        }
    }

    if (partial) {
        // row groups of this workgroup, added in index order
        constexpr int PER = O * K;
#pragma unroll
        for (int o = 0; o < O; ++o)
#pragma unroll
            for (int k = 0; k < K; ++k) lds[(rg * PER + o * K + k) * G + g] = acc[o][k];
        __syncthreads();
        if (rg == 0 && i_ok) {
            float* out = partial + (int64_t)blockIdx.x * I * O * K + (int64_t)i * O * K;
#pragma unroll
            for (int e = 0; e < PER; ++e) {
                float s = 0.0f;
                for (int q = 0; q < RPW; ++q) s += lds[(q * PER + e) * G + g];
                out[e] = s;
            }
        }
    }
}

// out[e] = sum_s partial[s][e], slices added in a fixed order: GROUPS slice groups take
// every GROUPS-th slice each, then the group sums are added in group order.
// block = 256 threads = GROUPS slice groups x 256/GROUPS elements; grid.x = ceil(n/(256/GROUPS)).
// Dynamic LDS: GROUPS x (256/GROUPS + 1) floats.
// The output may be a window of a larger tensor: element e goes to out[(e / run) * stride + e % run]
// (runs of `run` consecutive elements, `stride` apart); run = n writes out[e].
template <int GROUPS>
__global__ void __launch_bounds__(256)
sum_slices_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n, int n_slices, int64_t run,
                  int64_t stride)
{
    constexpr int EL = 256 / GROUPS;
    extern __shared__ __align__(16) float lds[];
    const int el = threadIdx.x % EL, sg = threadIdx.x / EL;
    const int64_t e = (int64_t)blockIdx.x * EL + el;
    float s = 0.0f;
    if (e < n) {
        const float* p = partial + (int64_t)sg * n + e;
        const int64_t step = (int64_t)GROUPS * n;
        int q = sg;
        // four slices per trip: the loads are issued together, the adds keep slice order
        for (; q + 3 * GROUPS < n_slices; q += 4 * GROUPS, p += 4 * step) {
            const float a0 = p[0], a1 = p[step], a2 = p[2 * step], a3 = p[3 * step];
            s += a0; s += a1; s += a2; s += a3;
        }
        for (; q < n_slices; q += GROUPS, p += step) s += p[0];
    }
    lds[sg * (EL + 1) + el] = s;
    __syncthreads();
    if (sg == 0 && e < n) {
        float total = 0.0f;
#pragma unroll
        for (int q = 0; q < GROUPS; ++q) total += lds[q * (EL + 1) + el];
        out[(e / run) * stride + e % run] = total;
    }
}

// The same sum for a few slices (up to 8): plain streaming, four consecutive elements per thread, slices
// added in slice order.  VEC = 4 when n is a multiple of 4 and both pointers are 16-byte aligned: every
// slice's run of four is then one 16-byte access.  grid.x = ceil(n / 1024).
template <int VEC>
__global__ void __launch_bounds__(256)
sum_few_slices_kernel(const float* __restrict__ partial, float* __restrict__ out, int64_t n, int n_slices)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (e >= n) return;
    if constexpr (VEC == 4) {
        f4 s = *reinterpret_cast<const f4*>(partial + e);
        for (int q = 1; q < n_slices; ++q) s += *reinterpret_cast<const f4*>(partial + (int64_t)q * n + e);
        *reinterpret_cast<f4*>(out + e) = s;
    } else {
        const int64_t end = e + 4 < n ? e + 4 : n;
        for (int64_t i = e; i < end; ++i) {
            float s = partial[i];
            for (int q = 1; q < n_slices; ++q) s += partial[(int64_t)q * n + i];
            out[i] = s;
        }
    }
}

}  // namespace chebykan
