// Forward pass of a whole narrow stack in one kernel.
//
// The paper evaluates three-layer stacks (Sec. 6.1, Table 2).  When every hidden width is at
// most 64, a 128-row tile of one layer's output is exactly the next layer's input tile, so a
// workgroup can carry its rows through all layers: each layer's output tile is written to
// HBM (the backward pass needs it) and kept in LDS, where the next layer's basis producer
// reads it instead of going back to HBM.  One launch replaces one per layer, and the narrow
// layers no longer pay a kernel start-up each.  Per layer the arithmetic is that of
// fwd_mfma_kernel (same tile, same chunk pipeline, 4 features per chunk); a last layer with
// 1..4 outputs is finished on the vector ALUs straight from the LDS tile.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_kernels.h"

namespace chebykan {

constexpr int CHAIN_MAX_LAYERS = 8;
constexpr int CHAIN_WIDTH = 64;          // widest hidden layer a chain can carry
constexpr int CHAIN_ACT_STRIDE = 65;     // floats per row of the LDS activation tile (odd: no bank conflicts)
constexpr int CHAIN_ACT_FLOATS = 128 * CHAIN_ACT_STRIDE;

struct ChainArgs {
    const float* C[CHAIN_MAX_LAYERS];     // coefficients of layer l, [width[l]][width[l+1]][K]
    float* act[CHAIN_MAX_LAYERS + 1];     // act[0] = input (read only), act[l+1] = output of layer l
    int width[CHAIN_MAX_LAYERS + 1];
    int n_layers;
};

template <int D>
using ChainCfg = FwdCfg<D, 64, 4, 4>;

template <int D>
constexpr int chain_lds_bytes() { return ChainCfg<D>::LDS_BYTES + CHAIN_ACT_FLOATS * 4; }

// One 128 x (<= 64) layer tile on the matrix cores.  Input rows come from HBM (FROM_LDS = false,
// x based at the tile's first row) or from the LDS activation tile; the output goes to y (HBM)
// and into the activation tile.  Ends with a barrier: the tile is complete and the stages are free.
template <int D, bool FROM_LDS>
__device__ __forceinline__ void chain_mfma_layer(const float* __restrict__ x, const float* __restrict__ C,
                                                 float* __restrict__ y, int rows_here, int I, int O,
                                                 float* lds, float* act)
{
    using Cfg = ChainCfg<D>;
    constexpr int K = Cfg::K, KP = Cfg::KP, BN = Cfg::BN, BI = Cfg::BI, VEC = Cfg::VEC;
    constexpr int SA = Cfg::SA, SS = Cfg::SS, TM = Cfg::TM, TN = Cfg::TN, WN = Cfg::WN;
    const ExactBasis basis(ExactBasis::Args{}, nullptr, K, 0, 0);
    const int t = threadIdx.x;

    const BufferView xv = make_view(x, FROM_LDS ? 0 : (int64_t)rows_here * I);
    const BufferView cv = make_view(C, (int64_t)I * O * K);
    const int xr_row = t >> 1;
    const int xr_f0 = (t & 1) * Cfg::XPT;
    const uint32_t x_off = (uint32_t)xr_row * (uint32_t)I + (uint32_t)xr_f0;
    const uint32_t OK_ = (uint32_t)O * (uint32_t)K;

    float xreg[Cfg::XPT];
    float creg[Cfg::NFULL * VEC + Cfg::NREM];

    auto load_chunk = [&](int i0) {
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            const int i = i0 + xr_f0 + j;
            if constexpr (FROM_LDS) {
                xreg[j] = i < I ? act[xr_row * CHAIN_ACT_STRIDE + i] : 0.0f;
            } else {
                const float v = load1(xv, x_off + (uint32_t)(i0 + j));
                xreg[j] = i < I ? v : 0.0f;
            }
        }
#pragma unroll
        for (int j = 0; j < Cfg::NFULL; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            const bufx4 v = load4(cv, (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K)));
            creg[j * 4 + 0] = v[0]; creg[j * 4 + 1] = v[1]; creg[j * 4 + 2] = v[2]; creg[j * 4 + 3] = v[3];
        }
#pragma unroll
        for (int j = 0; j < Cfg::NREM; ++j) {
            int e = Cfg::NFULL * VEC * MFMA_THREADS + t + j * MFMA_THREADS;
            if (e > Cfg::NE - 1) e = Cfg::NE - 1;
            creg[Cfg::NFULL * VEC + j] = load1(cv, (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K)));
        }
    };
    // A coefficient slab narrower than the 64-wide tile (O < 64) runs on into the next feature's
    // slab: those columns are computed and never stored.
    auto store_coeff = [&](float* sB, int e, float v) {
        const int il = e / (BN * K), rem = e % (BN * K);
        sB[il * SS + (rem / K) * KP + rem % K] = v;
    };
    auto store_chunk = [&](float* sA, float* sB) {
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            float T[D + 1];
            basis.template T<D>(xreg[j], T);
            store_run<K, true>(sA + xr_row * SA + (xr_f0 + j) * K, T);
        }
#pragma unroll
        for (int j = 0; j < Cfg::NFULL; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            if constexpr (KP == K) {
                floatx4 v = {creg[j * 4 + 0], creg[j * 4 + 1], creg[j * 4 + 2], creg[j * 4 + 3]};
                *reinterpret_cast<floatx4*>(sB + (e / (BN * K)) * SS + e % (BN * K)) = v;
            } else {
#pragma unroll
                for (int q = 0; q < VEC; ++q) store_coeff(sB, e + q, creg[j * VEC + q]);
            }
        }
#pragma unroll
        for (int j = 0; j < Cfg::NREM; ++j) {
            int e = Cfg::NFULL * VEC * MFMA_THREADS + t + j * MFMA_THREADS;
            if (e > Cfg::NE - 1) e = Cfg::NE - 1;
            store_coeff(sB, e, creg[Cfg::NFULL * VEC + j]);
        }
    };

    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, h = lane >> 5;
    const int aBase = (wm * 64 + l32) * SA + h * (BI / 2) * K;
    const int bBase = h * (BI / 2) * SS + (wn * WN + l32) * KP;

    floatx16 acc[TM][TN], total[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) { acc[i][j] = zero16(); total[i][j] = zero16(); }

    // Chunk loop as in fwd_mfma_kernel: the instruction order is laid down per step, operands are read
    // LA steps ahead as single LDS reads at immediate offsets, and the producer work of a chunk is a list
    // of items (LDS writes of chunk c+1, each followed by the load of chunk c+2 that refills its register).
    constexpr int NSTEP = Cfg::NSTEP, W = Cfg::W;
    constexpr int LA = W > 1 ? W : (LOOKAHEAD < NSTEP / 2 ? LOOKAHEAD : NSTEP / 2);
    static_assert(NSTEP % W == 0, "whole groups");
    float aop[NSTEP][TM], bop[NSTEP][TN];
    auto read_step = [&](const float* pA, const float* pB, int s) {
        if (s % W == 0) fwd_read_group<Cfg>(pA, pB, s / W, aop, bop);
    };
    constexpr int XPT = Cfg::XPT, NCO = Cfg::NFULL + Cfg::NREM, NITEM = 2 * (XPT + NCO);
    auto item = [&](float* sA, float* sB, int i0, int q) {
        if (q < XPT) {
            float T[D + 1];
            basis.template T<D>(xreg[q], T);
            store_run<K, true>(sA + xr_row * SA + (xr_f0 + q) * K, T);
        } else if (q < XPT + Cfg::NFULL) {
            const int j = q - XPT;
            const int e = (t + j * MFMA_THREADS) * VEC;
            if constexpr (KP == K) {
                floatx4 v = {creg[j * 4 + 0], creg[j * 4 + 1], creg[j * 4 + 2], creg[j * 4 + 3]};
                *reinterpret_cast<floatx4*>(sB + (e / (BN * K)) * SS + e % (BN * K)) = v;
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) store_coeff(sB, e + v, creg[j * VEC + v]);
            }
        } else if (q < XPT + NCO) {
            const int j = q - XPT - Cfg::NFULL;
            int e = Cfg::NFULL * VEC * MFMA_THREADS + t + j * MFMA_THREADS;
            if (e > Cfg::NE - 1) e = Cfg::NE - 1;
            store_coeff(sB, e, creg[Cfg::NFULL * VEC + j]);
        } else if (q < 2 * XPT + NCO) {
            const int j = q - XPT - NCO;
            const int i = i0 + xr_f0 + j;
            if constexpr (FROM_LDS) {
                xreg[j] = i < I ? act[xr_row * CHAIN_ACT_STRIDE + i] : 0.0f;
            } else {
                const float v = load1(xv, x_off + (uint32_t)(i0 + j));
                xreg[j] = i < I ? v : 0.0f;
            }
        } else if (q < 2 * XPT + NCO + Cfg::NFULL) {
            const int j = q - 2 * XPT - NCO;
            const int e = (t + j * MFMA_THREADS) * VEC;
            const bufx4 v = load4(cv, (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K)));
            creg[j * 4 + 0] = v[0]; creg[j * 4 + 1] = v[1]; creg[j * 4 + 2] = v[2]; creg[j * 4 + 3] = v[3];
        } else {
            const int j = q - 2 * XPT - NCO - Cfg::NFULL;
            int e = Cfg::NFULL * VEC * MFMA_THREADS + t + j * MFMA_THREADS;
            if (e > Cfg::NE - 1) e = Cfg::NE - 1;
            creg[Cfg::NFULL * VEC + j] = load1(cv, (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K)));
        }
    };

    const int n_chunks = (I + BI - 1) / BI;
    load_chunk(0);
    store_chunk(lds, lds + Cfg::A_FLOATS);
    load_chunk(BI);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();   // stage c is complete; every wave has finished reading stage c+1
        float* sA = lds + (c & 1) * Cfg::STAGE;
        float* nA = lds + ((c + 1) & 1) * Cfg::STAGE;
        const float* pA = sA + aBase;
        const float* pB = sA + Cfg::A_FLOATS + bBase;
        const int i_next = (c + 2) * BI;
#pragma unroll
        for (int s = 0; s < LA; ++s) read_step(pA, pB, s);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (s + LA < NSTEP) read_step(pA, pB, s + LA);
#pragma unroll
            for (int q = 0; q < NITEM; ++q)
                if (q * NSTEP / NITEM == s) item(nA, nA + Cfg::A_FLOATS, i_next, item_at(q, NITEM));
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = mfma32(aop[s][i], bop[s][j], acc[i][j]);
            __builtin_amdgcn_sched_barrier(0);
        }
        if ((c + 1) % Cfg::FOLD == 0) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) { total[i][j] += acc[i][j]; acc[i][j] = zero16(); }
        }
    }

    __syncthreads();   // every wave is done with the stages and with the activation tile it read
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const floatx16 v = total[i][j] + acc[i][j];
            const int col = wn * WN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = wm * 64 + i * 32 + mfma_row(r, h);
                act[row * CHAIN_ACT_STRIDE + col] = v[r];
                if (row < rows_here && col < O) y[(int64_t)row * O + col] = v[r];
            }
        }
    __syncthreads();   // the tile is complete for the next layer
}

// Last layer with O <= 4 outputs from the LDS tile: two threads per row take half of the
// input features each, the two halves are added in a fixed order.
template <int D, int O>
__device__ __forceinline__ void chain_narrow_tail(const float* __restrict__ C, float* __restrict__ y, int rows_here,
                                                  int I, const float* act)
{
    constexpr int K = D + 1;
    const ExactBasis basis(ExactBasis::Args{}, nullptr, K, 0, 0);
    const int t = threadIdx.x;
    const int row = t >> 1, half = t & 1;
    const int per = (I + 1) / 2;
    const int i_begin = half * per, i_end = (i_begin + per < I) ? i_begin + per : I;
    float sum[O];
#pragma unroll
    for (int o = 0; o < O; ++o) sum[o] = 0.0f;
    for (int i = i_begin; i < i_end; ++i) {
        float T[K];
        basis.template T<D>(act[row * CHAIN_ACT_STRIDE + i], T);
        const float* c = C + (int64_t)i * O * K;
#pragma unroll
        for (int o = 0; o < O; ++o) {
            float s = 0.0f;
#pragma unroll
            for (int k = 0; k < K; ++k) s = fmaf(c[o * K + k], T[k], s);
            sum[o] += s;
        }
    }
#pragma unroll
    for (int o = 0; o < O; ++o) {
        const float other = __shfl_xor(sum[o], 1);
        const float lo = half == 0 ? sum[o] : other, hi = half == 0 ? other : sum[o];
        if (half == 0 && row < rows_here) y[(int64_t)row * O + o] = lo + hi;
    }
}

// grid.x = ceil(B / 128).  Dynamic LDS: chain_lds_bytes<D>().
template <int D>
__global__ void __launch_bounds__(MFMA_THREADS, 2) fwd_chain_kernel(ChainArgs a, int B)
{
    extern __shared__ __align__(16) float lds[];
    float* act = lds + ChainCfg<D>::LDS_BYTES / 4;
    const int b0 = blockIdx.x * 128;
    const int rows_here = B - b0 < 128 ? B - b0 : 128;
    for (int l = 0; l < a.n_layers; ++l) {
        const int I = a.width[l], O = a.width[l + 1];
        float* y = a.act[l + 1] + (int64_t)b0 * O;
        const bool narrow_last = l == a.n_layers - 1 && l > 0 && O <= 4;
        if (narrow_last) {
            switch (O) {
                case 1: chain_narrow_tail<D, 1>(a.C[l], y, rows_here, I, act); break;
                case 2: chain_narrow_tail<D, 2>(a.C[l], y, rows_here, I, act); break;
                case 3: chain_narrow_tail<D, 3>(a.C[l], y, rows_here, I, act); break;
                default: chain_narrow_tail<D, 4>(a.C[l], y, rows_here, I, act); break;
            }
        } else if (l == 0) {
            chain_mfma_layer<D, false>(a.act[0] + (int64_t)b0 * I, a.C[l], y, rows_here, I, O, lds, act);
        } else {
            chain_mfma_layer<D, true>(nullptr, a.C[l], y, rows_here, I, O, lds, act);
        }
    }
}

}  // namespace chebykan
