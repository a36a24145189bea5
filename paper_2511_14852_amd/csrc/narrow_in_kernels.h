// Backward pass of a layer with very few inputs (in * (degree+1) <= 64, out <= 64) in one kernel.
//
// Such a layer (the first layer of a tabular network: 8 features) has one (i,k) tile and one
// output tile.  Its two gradients read the same dy rows, and the general kernels each spend
// most of their time starting up, so here one workgroup takes a slice of rows and per chunk
// of 32 rows computes BOTH
//     dC partial  += Phi^T * dy          (64 x 64 block; paper Alg. 2, coeff_grad)
//     G = dy * W^T, dx = (1-u^2) sum_k G T_k'   (32 x 64 block; paper Alg. 2, x_grad)
// from one staged dy tile: 32 MFMAs per wave and chunk, none of them wasted on padding
// rows.  W[(i,k)][o] = C[i][o][k] stays in LDS for the whole workgroup.  The partials go to the
// workspace in the layout of dC_mfma_kernel and are added by dC_combine_kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_kernels.h"

namespace chebykan {

constexpr int NIN_M = 64;          // (i,k) rows of the tile
constexpr int NIN_O = 64;          // output columns of the tile
constexpr int NIN_ROWS = 32;       // batch rows per chunk
constexpr int NIN_S = 65;          // odd LDS row stride: row-wise and column-wise operand reads are conflict free
constexpr int NIN_W_FLOATS = NIN_M * NIN_S;
constexpr int NIN_STAGE_FLOATS = 2 * NIN_ROWS * NIN_S;     // Phi^T tile + dy tile
constexpr int NIN_G_FLOATS = 2 * NIN_ROWS * NIN_S;         // two partial G tiles (one per half of the outputs)
constexpr int NIN_LDS_BYTES = (NIN_W_FLOATS + 2 * NIN_STAGE_FLOATS + NIN_G_FLOATS) * 4;

// One workgroup = one batch slice.  dx or partial may be null (that gradient is skipped).
template <int D, class Basis = ExactBasis>
__device__ __forceinline__ void bwd_narrow_in_body(const float* __restrict__ x, const float* __restrict__ C,
                                                   const float* __restrict__ dy, float* __restrict__ dx,
                                                   float* __restrict__ partial, int B, int I, int O, int rows_per_slice,
                                                   typename Basis::Args bargs, int slice)
{
    constexpr int K = D + 1, S = NIN_S;
    constexpr int EPT = 2;   // (row, feature) elements per thread and chunk: 32 * I <= 32 * 16
    extern __shared__ __align__(16) float lds[];
    float* sW = lds;
    float* sStage = lds + NIN_W_FLOATS;
    float* sG = sStage + 2 * NIN_STAGE_FLOATS;
    const Basis basis(bargs, lds + NIN_LDS_BYTES / 4, K, (int)threadIdx.x, MFMA_THREADS);

    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int IK = I * K;
    const int64_t r_begin = (int64_t)slice * rows_per_slice;
    int64_t r_end = r_begin + rows_per_slice;
    if (r_end > B) r_end = B;
    const int n_rows = r_end > r_begin ? (int)(r_end - r_begin) : 0;
    const int n_chunks = (n_rows + NIN_ROWS - 1) / NIN_ROWS;

    // views over this slice: rows past its end read as zero (zero dy adds nothing to dC)
    const BufferView xv = make_view(x + r_begin * I, (int64_t)n_rows * I);
    const BufferView gv = make_view(dy + r_begin * O, (int64_t)n_rows * O);

    // W[(i,k)][o] = C[i][o][k], zero outside the real rows and columns
    for (int e = t; e < NIN_M * NIN_O; e += MFMA_THREADS) {
        const int m = e / NIN_O, o = e % NIN_O;
        sW[m * S + o] = (m < IK && o < O) ? C[((int64_t)(m / K) * O + o) * K + m % K] : 0.0f;
    }

    // producer state: this thread's (row, feature) elements of a chunk
    float xreg[EPT], greg[8];
    float slope_cur[EPT], slope_nxt[EPT];
    float dT_cur[EPT][D > 0 ? D : 1], dT_nxt[EPT][D > 0 ? D : 1];
    const int n_el = NIN_ROWS * I;

    auto load_chunk = [&](int c) {
        const uint32_t row0 = (uint32_t)c * NIN_ROWS;
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int e = t + j * MFMA_THREADS;
            const int ec = e < n_el ? e : n_el - 1;
            xreg[j] = load1(xv, row0 * (uint32_t)I + (uint32_t)ec);      // element e of the chunk = (row e / I, feature e % I)
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = t + j * MFMA_THREADS;                           // (row e / 64, column e % 64)
            const int o = e % NIN_O;
            const float v = load1(gv, (row0 + (uint32_t)(e / NIN_O)) * (uint32_t)O + (uint32_t)o);
            greg[j] = o < O ? v : 0.0f;                                   // a column past O would be the next row
        }
    };
    auto store_chunk = [&](float* sPhi, float* sDy) {
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            const int e = t + j * MFMA_THREADS;
            if (e < n_el) {
                const int row = e / I, i = e % I;
                float T[K];
                basis.template T_dT<D>(xreg[j], T, dT_nxt[j], slope_nxt[j], true);
                float* dst = sPhi + row * S + i * K;
#pragma unroll
                for (int k = 0; k < K; ++k) dst[k] = T[k];
            }
        }
        // columns of the Phi^T tile past I*K feed output rows that are never stored; keep them finite
        for (int e = t; e < NIN_ROWS * (NIN_M - IK); e += MFMA_THREADS)
            sPhi[(e / (NIN_M - IK)) * S + IK + e % (NIN_M - IK)] = 0.0f;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = t + j * MFMA_THREADS;
            sDy[(e / NIN_O) * S + e % NIN_O] = greg[j];
        }
    };

    // consumer roles: dC block (mb, ob) of the 64 x 64 tile; G block nb over the output half oh
    const int mb = wave >> 1, ob = wave & 1;
    const int nb = wave & 1, oh = wave >> 1;
    floatx16 accC = zero16(), totC = zero16();

    load_chunk(0);
    store_chunk(sStage, sStage + NIN_ROWS * S);
#pragma unroll
    for (int j = 0; j < EPT; ++j) {
        slope_cur[j] = slope_nxt[j];
#pragma unroll
        for (int k = 0; k < D; ++k) dT_cur[j][k] = dT_nxt[j][k];
    }
    load_chunk(1);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();   // stage c (and W) complete; the previous chunk's epilogue is over
        const float* sPhi = sStage + (c & 1) * NIN_STAGE_FLOATS;
        const float* sDy = sPhi + NIN_ROWS * S;
        float* nPhi = sStage + ((c + 1) & 1) * NIN_STAGE_FLOATS;
        if (partial) {
#pragma unroll
            for (int s = 0; s < NIN_ROWS / 2; ++s) {
                const float a = sPhi[(2 * s + h) * S + mb * 32 + l32];
                const float b = sDy[(2 * s + h) * S + ob * 32 + l32];
                accC = mfma32(a, b, accC);
            }
        }
        if (dx) {
            floatx16 accG = zero16();
#pragma unroll
            for (int s = 0; s < NIN_O / 4; ++s) {
                const int o = oh * 32 + 2 * s + h;
                const float a = sDy[l32 * S + o];
                const float b = sW[(nb * 32 + l32) * S + o];
                accG = mfma32(a, b, accG);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) sG[(oh * NIN_ROWS + mfma_row(r, h)) * S + nb * 32 + l32] = accG[r];
        }
        store_chunk(nPhi, nPhi + NIN_ROWS * S);
        load_chunk(c + 2);
        if ((c + 1) % (FOLD_TERMS / NIN_ROWS) == 0) { totC += accC; accC = zero16(); }
        __syncthreads();   // the two partial G tiles are complete
        if (dx) {
#pragma unroll
            for (int j = 0; j < EPT; ++j) {
                const int e = t + j * MFMA_THREADS;
                const int row = e / I, i = e % I;
                if (e < n_el && c * NIN_ROWS + row < n_rows) {
                    const float* g0 = sG + row * S + i * K;
                    const float* g1 = g0 + NIN_ROWS * S;
                    float sum = 0.0f;
#pragma unroll
                    for (int k = 1; k <= D; ++k) sum = fmaf(g0[k] + g1[k], dT_cur[j][k - 1], sum);
                    dx[(r_begin + c * NIN_ROWS + row) * I + i] = slope_cur[j] * sum;
                }
            }
        }
#pragma unroll
        for (int j = 0; j < EPT; ++j) {
            slope_cur[j] = slope_nxt[j];
#pragma unroll
            for (int k = 0; k < D; ++k) dT_cur[j][k] = dT_nxt[j][k];
        }
    }

    if (partial) {
        float* out = partial + (int64_t)slice * IK * O;
        const floatx16 v = totC + accC;
        const int col = ob * 32 + l32;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = mb * 32 + mfma_row(r, h);
            if (m < IK && col < O) out[(int64_t)m * O + col] = v[r];
        }
    }
}

// grid.x = n_slices.
template <int D, class Basis = ExactBasis>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
bwd_narrow_in_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                     float* __restrict__ dx, float* __restrict__ partial, int B, int I, int O, int rows_per_slice,
                     typename Basis::Args bargs)
{
    bwd_narrow_in_body<D, Basis>(x, C, dy, dx, partial, B, I, O, rows_per_slice, bargs, (int)blockIdx.x);
}

// Two independent operations of a stack's backward pass in ONE launch: the coefficient gradient of
// layer l (matrix-core slices, see dC_mfma_kernel) and the whole backward pass of the few-inputs
// layer l-1 below it.  Both only need dx of layer l, which an earlier kernel wrote; neither reads what
// the other writes.  Sharing a launch lets their start-up and wind-down phases overlap and puts
// workgroups of the vector-ALU-heavy and of the MFMA-heavy operation on the same compute units.
// The first n_first workgroups take the few-inputs layer (the longer-running ones first).
struct DcSliceArgs {
    const float* x;
    const float* dy;
    float* partial;
    int B, I, O, n_tiles_o, o_begin, n_tiles_i, n_slices, rows_per_slice;
};
struct FewInputsArgs {
    const float* x;
    const float* C;
    const float* dy;
    float* dx;
    float* partial;
    int B, I, O, rows_per_slice;
};
template <class DcCfgT, int D>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
dC_with_few_inputs_kernel(DcSliceArgs a, FewInputsArgs b, int n_first)
{
    if ((int)blockIdx.x < n_first)
        bwd_narrow_in_body<D, ExactBasis>(b.x, b.C, b.dy, b.dx, b.partial, b.B, b.I, b.O, b.rows_per_slice, ExactBasis::Args{},
                                          (int)blockIdx.x);
    else
        dC_mfma_body<DcCfgT, ExactBasis>(a.x, a.dy, a.partial, a.B, a.I, a.O, a.n_tiles_o, a.o_begin, a.n_tiles_i, a.n_slices,
                                         a.rows_per_slice, ExactBasis::Args{}, nullptr, (int)blockIdx.x - n_first);
}

}  // namespace chebykan
