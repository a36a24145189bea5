// fp32 MFMA kernels of the Chebyshev-KAN layer for gfx950 (wave64).
//
// The layer is three dense contractions around an on-the-fly basis
// Phi[b,(i,k)] = T_k(tanh x[b,i])  (never written to HBM):
//
//   forward   y  = Phi * W              M = b, N = o,      contraction over (i,k)
//   dC        dC = Phi^T * dy           M = (i,k), N = o,  contraction over b
//   dx        G  = dy * W^T             M = b, N = (i,k),  contraction over o
//             dx[b,i] = (1-u^2) sum_k G[b,(i,k)] T_k'(u)
//
// with W[(i,k),o] = C[i,o,k] (paper Eq. 2-3, Alg. 1-2).  Each workgroup of 256
// threads (4 waves, 2 x 2) owns a 128-row output tile, stages both operands of
// one contraction chunk in LDS (double buffered, one barrier per chunk) and
// feeds v_mfma_f32_32x32x2_f32.  Coefficients are read in their original
// [in][out][degree+1] layout: for one input feature a run of outputs is one
// contiguous slab, so global loads are unit-stride without any repacking pass;
// the k/o transposition happens in the LDS addressing.
//
// Accuracy: accumulators are folded into a second set about every 512
// contraction terms, so that long fp32 sums keep a relative error near 1e-6.
//
// Chunk loops: fp32 MFMA and vector-ALU instructions do not overlap on this chip, so beyond its
// MFMAs a loop costs what vector-ALU instructions and stalls it holds.  The bodies are written one
// step at a time - a step is the set of independent MFMAs that share operands, closed by a
// scheduling fence - with each step's share of operand reads, LDS writes and global loads next to
// it in the source, operand offsets as instruction immediates, and masking of ragged ends confined
// to the last chunks.
//
// MFMA operand layout used throughout (32x32x2, lane l, half h = l/32):
//   A: lane supplies A[row = l%32][k = h];  B: lane supplies B[k = h][col = l%32];
//   D: register r holds D[row = 8*(r/4) + 4*h + r%4][col = l%32].
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "basis.h"
#include "buffer_io.h"

// Hides a value from the optimiser at one point of the program (emits no instruction); a host-side
// build of the kernels may define it away.
#ifndef CHEBYKAN_OPAQUE
#define CHEBYKAN_OPAQUE(v) asm volatile("" : "+v"(v))
#endif

// Optional in-kernel time stamps for profiling builds (slot 0 kernel entry, 1 before the
// chunk loop, 2 after it, 3 kernel exit); compiled out unless the includer defines it.
#ifndef CHEBYKAN_PROBE
#define CHEBYKAN_PROBE(slot)
#endif

namespace chebykan {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int MFMA_THREADS = 256;
constexpr int FOLD_TERMS = 512;  // contraction terms between accumulator folds
constexpr int LOOKAHEAD = 2;     // MFMA steps between an LDS operand read and its use

__device__ __forceinline__ floatx16 mfma32(float a, float b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ floatx16 zero16()
{
    floatx16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.0f;
    return z;
}

// One MFMA operand from LDS.  The access is volatile so that it stays a single 4-byte read whose
// constant offset goes into the instruction's 16-bit offset field: left to itself the compiler pairs
// operand reads into two-address reads, whose offsets reach only 1 KB, and pays for the pairing with
// a vector add per new base - and every vector-ALU instruction in a chunk loop takes time from the
// matrix pipe, while an LDS instruction only takes an issue slot.
#ifndef CHEBYKAN_LDS_OPERAND
#define CHEBYKAN_LDS_OPERAND(p) (*(const volatile __attribute__((address_space(3))) float*)(p))
#endif
__device__ __forceinline__ float lds_operand(const float* p) { return CHEBYKAN_LDS_OPERAND(p); }
#ifndef CHEBYKAN_LDS_STORE
#define CHEBYKAN_LDS_STORE(p, v) (*(volatile __attribute__((address_space(3))) float*)(p) = (v))
#endif

// The producer work of a chunk is a list of n items: n/2 LDS writes of the next chunk's data, held in
// registers, then the n/2 global loads that refill those registers with the chunk after.  item_at gives
// the p-th item to issue: write 0, load 0, write 1, load 1, ... - each load follows the write that
// frees its register, and is consumed a whole chunk later.
__host__ __device__ constexpr int item_at(int p, int n) { return p % 2 == 0 ? p / 2 : n / 2 + p / 2; }

// row inside a 32x32 MFMA output block held by register r of a lane in half h
__device__ __forceinline__ int mfma_row(int r, int h) { return 8 * (r >> 2) + 4 * h + (r & 3); }

// ============================================================== forward
template <int W> struct LdsVec;
template <> struct LdsVec<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct LdsVec<4> { typedef float type __attribute__((ext_vector_type(4))); };

// K consecutive floats to LDS.  SINGLE: one 4-byte write each at an immediate offset, through volatile
// accesses so that they stay that way - where rows are 8- or 16-byte aligned the compiler otherwise
// merges them into wide writes, for which the values first have to be moved into consecutive
// registers, and only vector-ALU instructions take time from the MFMAs.
template <int K, bool SINGLE>
__device__ __forceinline__ void store_run(float* dst, const float (&v)[K])
{
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if constexpr (SINGLE) CHEBYKAN_LDS_STORE(dst + k, v[k]);
        else dst[k] = v[k];
    }
}

// Operands of the W steps of group g of a forward chunk (see FwdCfg::W): pA / pB are the lane's bases
// in the Phi tile and the coefficient tile.
template <class Cfg>
__device__ __forceinline__ void fwd_read_group(const float* pA, const float* pB, int g, float (&aop)[Cfg::NSTEP][Cfg::TM],
                                               float (&bop)[Cfg::NSTEP][Cfg::TN])
{
    constexpr int W = Cfg::W, K = Cfg::K;
    const int s0 = W * g, ih = s0 / K, k0 = s0 % K;      // a group never straddles two features: W divides K
    if constexpr (W > 1) {
        typedef typename LdsVec<W>::type vec;
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i) {
            const vec a = *reinterpret_cast<const vec*>(pA + i * 32 * Cfg::SA + s0);
#pragma unroll
            for (int w = 0; w < W; ++w) aop[s0 + w][i] = a[w];
        }
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) {
            const vec b = *reinterpret_cast<const vec*>(pB + ih * Cfg::SS + j * 32 * Cfg::KP + k0);
#pragma unroll
            for (int w = 0; w < W; ++w) bop[s0 + w][j] = b[w];
        }
    } else {
#pragma unroll
        for (int i = 0; i < Cfg::TM; ++i) aop[s0][i] = lds_operand(pA + i * 32 * Cfg::SA + s0);
#pragma unroll
        for (int j = 0; j < Cfg::TN; ++j) bop[s0][j] = lds_operand(pB + ih * Cfg::SS + j * 32 * Cfg::KP + k0);
    }
}

// RB_ = 32-row blocks of the tile that can hold real rows.  4: the waves form a 2 x 2 grid
// (64 rows x BN/2 outputs each).  1 or 2 (a batch of at most 32 or 64 rows, BN = 128): the four
// waves stand side by side, 32 outputs each, and issue no MFMA for row blocks that are all padding.
template <int D_, int BN_, int BI_, int VEC_, int RB_ = 4>
struct FwdCfg {
    static constexpr int D = D_, K = D_ + 1;
    // W = contraction steps fetched by one LDS read of an operand.  A lane's operands of consecutive steps
    // are consecutive in LDS on both sides (its Phi row; the K coefficients of one feature and output), so
    // where K is 4 or 6 they are read 16 or 8 bytes at a time: rows and runs then start on such
    // boundaries (KP = K: the coefficient runs are copied verbatim) and strides are odd multiples of W
    // floats, which spreads a pass of 16-byte (8 lanes) or 8-byte (16 lanes) accesses over all banks.
    // Otherwise single reads and odd strides.
    static constexpr int W = K == 4 ? 4 : (K == 6 ? 2 : 1);
    static constexpr int KP = W > 1 ? K : (K | 1);             // per-output stride in LDS
    static constexpr int BM = 128, BN = BN_, BI = BI_, VEC = VEC_, RB = RB_;
    static constexpr int WN = RB == 4 ? BN / 2 : BN / 4, TM = RB == 4 ? 2 : RB, TN = WN / 32;
    static_assert(RB == 4 || ((RB == 1 || RB == 2) && BN == 128), "small-batch tiles are 128 outputs wide");
    static constexpr int CH = BI * K;                          // contraction terms per chunk
    static constexpr int SA = W > 1 ? CH + ((CH / W) % 2 == 0 ? W : 2 * W) : (CH | 1);   // row stride of the Phi tile
    static constexpr int SS = BN * KP;                         // stride between feature slabs
    static constexpr int A_FLOATS = (BM * SA + 3) & ~3;
    static constexpr int B_FLOATS = (BI * SS + 3) & ~3;
    static constexpr int STAGE = A_FLOATS + B_FLOATS;
    static constexpr int LDS_BYTES = 2 * STAGE * 4;
    static constexpr int NSTEP = (BI / 2) * K;
    static constexpr int FOLD = (FOLD_TERMS / CH) > 0 ? (FOLD_TERMS / CH) : 1;
    static constexpr int XPT = BI / 2;                         // x values per thread per chunk
    static constexpr int NE = BI * BN * K;                     // coefficient floats per chunk
    // every thread loads NFULL vectors of VEC floats plus NREM single floats: no ragged round
    static constexpr int NFULL = NE / (VEC * MFMA_THREADS);
    // (a last partial round repeats the final element in the idle threads: same value, same place)
    static constexpr int NREM = (NE - NFULL * VEC * MFMA_THREADS + MFMA_THREADS - 1) / MFMA_THREADS;
    static constexpr int NMFMA = NSTEP * TM * TN;              // MFMA instructions per chunk and wave
    // producer work spread over the chunk's steps, or all of it ahead of the MFMAs (see DcCfg; for this
    // kernel no difference was measured at either width)
    static constexpr bool CLUSTER = false;
    static_assert(VEC == 4, "coefficient runs are copied 16 bytes at a time");
    static_assert(BI % 2 == 0 && BN % 64 == 0, "tile shape");
    static_assert(W == 1 || (CH % W == 0 && (SA / W) % 2 == 1 && ((BI / 2) * K) % W == 0 && K % W == 0), "wide operand reads");
    static_assert((BN * K) % VEC == 0, "vector width");
};

// y[b,o] = sum_i sum_k C[i,o,k] T_k(tanh x[b,i])      (paper Eq. 2-3; Alg. 1 as a function)
// grid.x = ceil(B/128) * n_tiles_o, output-tile index fastest; grid.y = contraction ranges.
// The launch covers the n_tiles_o BN-wide output tiles that start at column o_begin, so a width
// just above a multiple of 128 can be tiled with 128-wide tiles plus one 64-wide tile.
//
// Per chunk c: barrier; the MFMA steps of chunk c, and between them chunk c+1 generated into the
// other LDS stage and chunk c+2 requested from HBM.  All loads go through bounds-checked buffer
// views (zeros beyond the tensor), so this body has no branches.
template <class Cfg, class Basis = ExactBasis>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
fwd_mfma_kernel(const float* __restrict__ x, const float* __restrict__ C, float* __restrict__ y,
                int B, int I, int O, int n_tiles_o, int o_begin, int chunks_per_split, typename Basis::Args bargs)
{
    constexpr int D = Cfg::D, K = Cfg::K, KP = Cfg::KP, BN = Cfg::BN, BI = Cfg::BI, VEC = Cfg::VEC;
    constexpr int SA = Cfg::SA, SS = Cfg::SS, TM = Cfg::TM, TN = Cfg::TN, WN = Cfg::WN;
    extern __shared__ __align__(16) float lds[];
    CHEBYKAN_PROBE(0);
    const Basis basis(bargs, lds + Cfg::LDS_BYTES / 4, Cfg::K, (int)threadIdx.x, MFMA_THREADS);

    const int t = threadIdx.x;
    const int tile_o = blockIdx.x % n_tiles_o;
    const int tile_b = blockIdx.x / n_tiles_o;
    const int b0 = tile_b * Cfg::BM;
    const int o0 = o_begin + tile_o * BN;   // a launch covers the BN-wide tiles from column o_begin on

    // --- producer role.  Views are based at this tile so that 32-bit offsets suffice.
    const int rows_here = B - b0 < Cfg::BM ? B - b0 : Cfg::BM;
    const BufferView xv = make_view(x + (int64_t)b0 * I, (int64_t)rows_here * I);
    // Coefficient view from this tile's first output to the end of the tensor: features past
    // I fall outside and read as zero.  A partial output tile reads into the next feature's
    // slab; those columns are never stored.
    const BufferView cv = make_view(C + (int64_t)o0 * K, (int64_t)I * O * K - (int64_t)o0 * K);
    const int xr_row = t >> 1;                     // row of the tile this thread generates basis for
    const int xr_f0 = (t & 1) * Cfg::XPT;          // first feature (inside the chunk)
    const uint32_t x_off = (uint32_t)xr_row * (uint32_t)I + (uint32_t)xr_f0;
    const uint32_t OK_ = (uint32_t)O * (uint32_t)K;

    float xreg[Cfg::XPT];
    float creg[Cfg::NFULL * VEC + Cfg::NREM];

    auto load_chunk = [&](int i0) {
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            // a feature index past I would read the next row: keep that out of the basis
            const float v = load1(xv, x_off + (uint32_t)(i0 + j));
            xreg[j] = (i0 + xr_f0 + j < I) ? v : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < Cfg::NFULL; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            const uint32_t off = (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K));
            if constexpr (VEC == 4) {
                const bufx4 v = load4(cv, off);
                creg[j * 4 + 0] = v[0]; creg[j * 4 + 1] = v[1]; creg[j * 4 + 2] = v[2]; creg[j * 4 + 3] = v[3];
            } else {
                creg[j] = load1(cv, off);
            }
        }
#pragma unroll
        for (int j = 0; j < Cfg::NREM; ++j) {
            int e = Cfg::NFULL * VEC * MFMA_THREADS + t + j * MFMA_THREADS;
            if (e > Cfg::NE - 1) e = Cfg::NE - 1;
            creg[Cfg::NFULL * VEC + j] = load1(cv, (uint32_t)(i0 + e / (BN * K)) * OK_ + (uint32_t)(e % (BN * K)));
        }
    };

    auto store_coeff = [&](float* sB, int e, float v) {
        const int il = e / (BN * K), rem = e % (BN * K);
        sB[il * SS + (rem / K) * KP + rem % K] = v;
    };
    auto store_chunk = [&](float* sA, float* sB) {
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            float T[D + 1];
            basis.template T<D>(xreg[j], T);
            store_run<K, (Cfg::W > 1)>(sA + xr_row * SA + (xr_f0 + j) * K, T);
        }
#pragma unroll
        for (int j = 0; j < Cfg::NFULL; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            if constexpr (VEC == 4 && KP == K) {
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

    // --- consumer role
    const int lane = t & 63, wave = t >> 6;
    const int wm = Cfg::RB == 4 ? wave >> 1 : 0, wn = Cfg::RB == 4 ? wave & 1 : wave;
    const int l32 = lane & 31, h = lane >> 5;
    int aBase = (wm * 64 + l32) * SA + h * (BI / 2) * K;
    int bBase = h * (BI / 2) * SS + (wn * WN + l32) * KP;
    // one register each for the whole loop (the compiler would otherwise rebuild them from their parts per chunk)
    CHEBYKAN_OPAQUE(aBase);
    CHEBYKAN_OPAQUE(bBase);

    floatx16 acc[TM][TN], total[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) { acc[i][j] = zero16(); total[i][j] = zero16(); }

    // The instruction order of a chunk is laid down by hand, one step (TM x TN independent MFMAs) at a
    // time with a scheduling fence after each.  Operands of a step are read LA steps ahead of the
    // MFMAs that use them, as single 4-byte reads at immediate offsets (see lds_operand).
    // Where a lane's operands are read several steps at a time (FwdCfg::W), a group of W steps is read
    // one group ahead.
    constexpr int NSTEP = Cfg::NSTEP, W = Cfg::W;
    constexpr int LA = W > 1 ? W : (LOOKAHEAD < NSTEP / 2 ? LOOKAHEAD : NSTEP / 2);
    static_assert(NSTEP % W == 0, "whole groups");
    float aop[NSTEP][TM], bop[NSTEP][TN];
    auto read_step = [&](const float* pA, const float* pB, int s) {
        if (s % W == 0) fwd_read_group<Cfg>(pA, pB, s / W, aop, bop);
    };
    // Producer work of a chunk as a list of items: the basis of this thread's XPT elements of chunk c+1,
    // the coefficient vectors and single floats of chunk c+1, then the loads of chunk c+2 into the same
    // registers.
    constexpr int XPT = Cfg::XPT, NCO = Cfg::NFULL + Cfg::NREM, NITEM = 2 * (XPT + NCO);
    auto item = [&](float* sA, float* sB, int i0, int q) {
        if (q < XPT) {
            float T[D + 1];
            basis.template T<D>(xreg[q], T);
            store_run<K, (Cfg::W > 1)>(sA + xr_row * SA + (xr_f0 + q) * K, T);
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
            // a feature index past I would read the next row: keep that out of the basis
            const float v = load1(xv, x_off + (uint32_t)(i0 + j));
            xreg[j] = (i0 + xr_f0 + j < I) ? v : 0.0f;
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

    // Chunks past the last one are loaded and stored too: their views return zeros and the
    // stage they land in is never read.  That keeps the loop body free of conditions.
    // blockIdx.y selects a range of chunks (a split contraction writes partial outputs, one
    // [B,O] plane per range, that a second kernel adds in range order)
    const int n_chunks_all = (I + BI - 1) / BI;
    const int c_begin = blockIdx.y * chunks_per_split;
    const int n_chunks = n_chunks_all - c_begin < chunks_per_split ? n_chunks_all - c_begin : chunks_per_split;
    y += (int64_t)blockIdx.y * B * O;
    load_chunk(c_begin * BI);
    store_chunk(lds, lds + Cfg::A_FLOATS);
    load_chunk((c_begin + 1) * BI);
    CHEBYKAN_PROBE(1);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();   // stage c is complete; every wave has finished reading stage c+1
        float* sA = lds + (c & 1) * Cfg::STAGE;
        float* nA = lds + ((c + 1) & 1) * Cfg::STAGE;
        const float* pA = sA + aBase;
        const float* pB = sA + Cfg::A_FLOATS + bBase;
        const int i_next = (c_begin + c + 2) * BI;
#pragma unroll
        for (int s = 0; s < LA; ++s) read_step(pA, pB, s);
        if constexpr (Cfg::CLUSTER) {
#pragma unroll
            for (int q = 0; q < NITEM; ++q) item(nA, nA + Cfg::A_FLOATS, i_next, item_at(q, NITEM));
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (s + LA < NSTEP) read_step(pA, pB, s + LA);
            if constexpr (!Cfg::CLUSTER) {
#pragma unroll
                for (int q = 0; q < NITEM; ++q)
                    if (q * NSTEP / NITEM == s) item(nA, nA + Cfg::A_FLOATS, i_next, item_at(q, NITEM));
            }
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
    CHEBYKAN_PROBE(2);

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const floatx16 v = total[i][j] + acc[i][j];
            const int col = o0 + wn * WN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = b0 + wm * 64 + i * 32 + mfma_row(r, h);
                if (row < B && col < O) y[(int64_t)row * O + col] = v[r];
            }
        }
    CHEBYKAN_PROBE(3);
}

// =================================================== coefficient gradient
template <int D_, int BN_, int VEC_, int BIC_ = 128 / (D_ + 1)>
struct DcCfg {
    static constexpr int D = D_, K = D_ + 1, BN = BN_, VEC = VEC_;
    static constexpr int BIC = BIC_;                    // input features per tile
    static constexpr int BMR = BIC * K;                 // real rows (i,k) of the 128-row tile
    static constexpr int BB = 32;                       // batch rows per chunk
    static constexpr int SMA = 128 + (BMR % 32);        // Phi^T tile row stride (see store below)
    static constexpr int SNB = BN;
    static constexpr int WN = BN / 2, TM = 2, TN = WN / 32;
    static constexpr int A_FLOATS = BB * SMA;
    static constexpr int B_FLOATS = BB * SNB;
    static constexpr int STAGE = (A_FLOATS + B_FLOATS + 3) & ~3;
    static constexpr int LDS_BYTES = 2 * STAGE * 4;
    static constexpr int NSTEP = BB / 2;
    static constexpr int FOLD = FOLD_TERMS / BB;
    // Where the producer work of a chunk goes: spread over the chunk's steps, or (64-wide tiles: two
    // accumulators per wave, where every interruption of the MFMA stream costs more) all of it ahead
    // of one uninterrupted run of MFMAs.  Measured both ways at both widths.
    static constexpr bool CLUSTER = BN == 64;
    static constexpr int NEA = BB * BIC;
    static constexpr int XPT = (NEA + MFMA_THREADS - 1) / MFMA_THREADS;
    static constexpr int NEB = BB * BN;
    static constexpr int GPT = NEB / VEC / MFMA_THREADS;
    static_assert(VEC == 4 && NEB % (VEC * MFMA_THREADS) == 0, "dy tile must split evenly into 16-byte vectors");
    static_assert(A_FLOATS % 4 == 0, "dy tile must stay 16-byte aligned");
    static_assert(BIC >= 1 && BMR <= 128, "tile rows");
    // single-slice launches turn their tile to the caller's [i][o][k] layout in LDS: [feature][output][K|1]
    static constexpr int KP = K | 1;
    static constexpr int DIRECT_FLOATS = BIC * BN * KP;
    static constexpr int DIRECT_LDS_BYTES = DIRECT_FLOATS * 4 > LDS_BYTES ? DIRECT_FLOATS * 4 : LDS_BYTES;
};

// partial[s][(i,k)][o] = sum over the rows of batch slice s of T_k(tanh x[b,i]) dy[b,o]
// (paper Alg. 2, coeff_grad; the batch axis is split into slices whose partial sums a
// second kernel adds in a fixed order - the two-stage reduction of Sec. 4.4 in place
// of atomics).  grid.x = tiles_ik * tiles_o * n_slices.  Same chunk pipeline as the
// forward kernel: loads through buffer views based at the slice (rows past the slice
// read as zero dy, so they add nothing), producer work between MFMA issues.
// `block` is the workgroup's linear id inside this operation (blockIdx.x when the kernel runs alone).
template <class Cfg, class Basis = ExactBasis>
__device__ __forceinline__ void dC_mfma_body(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ partial,
                                             int B, int I, int O, int n_tiles_o, int o_begin, int n_tiles_i, int n_slices,
                                             int rows_per_slice, typename Basis::Args bargs, float* __restrict__ direct, int block)
{
    constexpr int D = Cfg::D, K = Cfg::K, BN = Cfg::BN, VEC = Cfg::VEC, BB = Cfg::BB, BIC = Cfg::BIC;
    constexpr int SMA = Cfg::SMA, SNB = Cfg::SNB, TM = Cfg::TM, TN = Cfg::TN, WN = Cfg::WN;
    extern __shared__ __align__(16) float lds[];
    CHEBYKAN_PROBE(0);
    const Basis basis(bargs, lds + Cfg::LDS_BYTES / 4, Cfg::K, (int)threadIdx.x, MFMA_THREADS);

    const int t = threadIdx.x;
    // Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.
    // All tiles of one batch slice read the same x and dy rows, so they are given ids that are
    // equal mod 8 and adjacent in time: the slice's rows then come from HBM once, not once per tile.
    const int n_tiles = n_tiles_o * n_tiles_i;
    int tile, slice;
    {
        const int L = block;
        const int full = (n_slices / 8) * 8;               // slices in complete groups of 8
        if (L < full * n_tiles) {
            const int group = L / (8 * n_tiles), rem = L % (8 * n_tiles);
            slice = group * 8 + rem % 8;
            tile = rem / 8;
        } else {                                           // last, incomplete group: plain order
            const int rem = L - full * n_tiles;
            slice = full + rem / n_tiles;
            tile = rem % n_tiles;
        }
    }
    const int tile_o = tile % n_tiles_o;
    const int tile_i = tile / n_tiles_o;
    const int i0 = tile_i * BIC;
    const int o0 = o_begin + tile_o * BN;
    const int64_t r_begin = (int64_t)slice * rows_per_slice;
    int64_t r_end = r_begin + rows_per_slice;
    if (r_end > B) r_end = B;
    const int64_t n_rows = r_end > r_begin ? r_end - r_begin : 0;

    // Views over this slice.  A feature index past I reads the next row of x and a column
    // past O the next row of dy: both only reach outputs that are never stored.
    const BufferView xv = make_view(x + r_begin * I + i0, n_rows * I - i0);
    const BufferView gv = make_view(dy + r_begin * O + o0, n_rows * O - o0);

    float xreg[Cfg::XPT];
    float greg[Cfg::GPT * VEC];
    // element of the Phi^T chunk this thread generates; past-the-end threads repeat the last one
    int xe[Cfg::XPT];
#pragma unroll
    for (int j = 0; j < Cfg::XPT; ++j) {
        const int e = t + j * MFMA_THREADS;
        xe[j] = e < Cfg::NEA ? e : Cfg::NEA - 1;
    }

    auto load_chunk = [&](int c) {
        const uint32_t row0 = (uint32_t)c * BB;
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            const int bl = xe[j] / BIC, il = xe[j] % BIC;
            xreg[j] = load1(xv, (row0 + (uint32_t)bl) * (uint32_t)I + (uint32_t)il);
        }
#pragma unroll
        for (int j = 0; j < Cfg::GPT; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            const uint32_t off = (row0 + (uint32_t)(e / BN)) * (uint32_t)O + (uint32_t)(e % BN);
            if constexpr (VEC == 4) {
                const bufx4 v = load4(gv, off);
                greg[j * 4 + 0] = v[0]; greg[j * 4 + 1] = v[1]; greg[j * 4 + 2] = v[2]; greg[j * 4 + 3] = v[3];
            } else {
                greg[j] = load1(gv, off);
            }
        }
    };

    auto store_chunk = [&](float* sA, float* sB) {
#pragma unroll
        for (int j = 0; j < Cfg::XPT; ++j) {
            const int bl = xe[j] / BIC, il = xe[j] % BIC;
            float T[D + 1];
            basis.template T<D>(xreg[j], T);
            // SMA = BMR (mod 32): consecutive elements land K words apart across row ends too.  At even K the
            // compiler would pair the writes into 8-byte ones (register moves): single writes there.
            store_run<K, (K % 2 == 0)>(sA + bl * SMA + il * K, T);
        }
#pragma unroll
        for (int j = 0; j < Cfg::GPT; ++j) {
            const int e = (t + j * MFMA_THREADS) * VEC;
            const int bl = e / BN, n = e % BN;
            if constexpr (VEC == 4) {
                floatx4 v = {greg[j * 4 + 0], greg[j * 4 + 1], greg[j * 4 + 2], greg[j * 4 + 3]};
                *reinterpret_cast<floatx4*>(sB + bl * SNB + n) = v;
            } else {
                sB[bl * SNB + n] = greg[j];
            }
        }
    };

    const int lane = t & 63, wave = t >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, h = lane >> 5;
    int aBase = h * (BB / 2) * SMA + wm * 64 + l32;
    int bBase = h * (BB / 2) * SNB + wn * WN + l32;
    // one register each for the whole loop (the compiler would otherwise rebuild them from their parts per chunk)
    CHEBYKAN_OPAQUE(aBase);
    CHEBYKAN_OPAQUE(bBase);

    floatx16 acc[TM][TN], total[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) { acc[i][j] = zero16(); total[i][j] = zero16(); }

    // The instruction order of a chunk is laid down by hand, one step (TM x TN independent MFMAs) at a
    // time with a scheduling fence after each.  Operands of a step are read LA steps ahead of the
    // MFMAs that use them, as single 4-byte reads at immediate offsets (see lds_operand).
    constexpr int NSTEP = Cfg::NSTEP;
    constexpr int LA = LOOKAHEAD;
    float aop[NSTEP][TM], bop[NSTEP][TN];
    auto read_step = [&](const float* pA, const float* pB, int s) {
#pragma unroll
        for (int i = 0; i < TM; ++i) aop[s][i] = lds_operand(pA + s * SMA + i * 32);
#pragma unroll
        for (int j = 0; j < TN; ++j) bop[s][j] = lds_operand(pB + s * SNB + j * 32);
    };
    // Producer work of a chunk as a list of items: item j < XPT evaluates the basis of this thread's
    // j-th element of chunk c+1 and writes it; the next GPT items write the dy vectors of chunk c+1;
    // then come the loads of chunk c+2 into the same registers.
    constexpr int XPT = Cfg::XPT, GPT = Cfg::GPT, NITEM = 2 * (XPT + GPT);
    static_assert((MFMA_THREADS * VEC) % BN == 0, "a thread's dy vectors lie whole rows apart");
    const int g_lds = ((t * VEC) / BN) * SNB + (t * VEC) % BN;                          // in the LDS tile
    const uint32_t g_off = (uint32_t)((t * VEC) / BN) * (uint32_t)O + (uint32_t)((t * VEC) % BN);   // in the dy rows of a chunk
    auto item = [&](float* sA, float* sB, int c, int q) {
        const uint32_t row0 = (uint32_t)(c + 2) * BB;
        if (q < XPT) {
            const int bl = xe[q] / BIC, il = xe[q] % BIC;
            float T[D + 1];
            basis.template T<D>(xreg[q], T);
            store_run<K, (K % 2 == 0)>(sA + bl * SMA + il * K, T);
        } else if (q < XPT + GPT) {
            // vector j of this thread: row (4t)/BN + j*(1024/BN), column (4t)%BN - one base, constant offsets
            const int j = q - XPT;
            floatx4 v = {greg[j * 4 + 0], greg[j * 4 + 1], greg[j * 4 + 2], greg[j * 4 + 3]};
            *reinterpret_cast<floatx4*>(sB + g_lds + j * (MFMA_THREADS * VEC / BN) * SNB) = v;
        } else if (q < 2 * XPT + GPT) {
            const int j = q - XPT - GPT;
            const int bl = xe[j] / BIC, il = xe[j] % BIC;
            xreg[j] = load1(xv, (row0 + (uint32_t)bl) * (uint32_t)I + (uint32_t)il);
        } else {
            const int j = q - 2 * XPT - GPT;
            const bufx4 v = load4(gv, (row0 + (uint32_t)(j * (MFMA_THREADS * VEC / BN))) * (uint32_t)O + g_off);
            greg[j * 4 + 0] = v[0]; greg[j * 4 + 1] = v[1]; greg[j * 4 + 2] = v[2]; greg[j * 4 + 3] = v[3];
        }
    };

    const int n_chunks = (int)((n_rows + BB - 1) / BB);
    load_chunk(0);
    store_chunk(lds, lds + Cfg::A_FLOATS);
    load_chunk(1);
    CHEBYKAN_PROBE(1);
    for (int c = 0; c < n_chunks; ++c) {
        __syncthreads();   // stage c is complete; every wave has finished reading stage c+1
        float* sA = lds + (c & 1) * Cfg::STAGE;
        float* nA = lds + ((c + 1) & 1) * Cfg::STAGE;
        const float* pA = sA + aBase;
        const float* pB = sA + Cfg::A_FLOATS + bBase;
#pragma unroll
        for (int s = 0; s < LA; ++s) read_step(pA, pB, s);
        if constexpr (Cfg::CLUSTER) {
#pragma unroll
            for (int q = 0; q < NITEM; ++q) item(nA, nA + Cfg::A_FLOATS, c, item_at(q, NITEM));
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            if (s + LA < NSTEP) read_step(pA, pB, s + LA);
            if constexpr (!Cfg::CLUSTER) {
#pragma unroll
                for (int q = 0; q < NITEM; ++q)
                    if (q * NSTEP / NITEM == s) item(nA, nA + Cfg::A_FLOATS, c, item_at(q, NITEM));
            }
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

    CHEBYKAN_PROBE(2);
    const int64_t IK = (int64_t)I * K;
    if (direct) {
        // One slice only (the host passes `direct` = dC then): the tile is final.  It goes through LDS
        // as [feature][output][K|1] and leaves as one contiguous run of outputs x K per feature - the
        // caller's [i][o][k] layout - so no partial tensor and no second kernel are needed.
        constexpr int KP = Cfg::KP;
        __syncthreads();   // every wave has finished reading the last stage
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const floatx16 v = total[i][j] + acc[i][j];
                const int col = wn * WN + j * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ml = wm * 64 + i * 32 + mfma_row(r, h);
                    if (ml < Cfg::BMR) lds[((ml / K) * BN + col) * KP + ml % K] = v[r];
                }
            }
        __syncthreads();
        const int cols_here = O - o0 < BN ? O - o0 : BN;
        bool copied = false;
        if constexpr (KP == K) {
            // odd K: the LDS tile is already the run, element for element; with O a multiple of 4 every
            // run starts 16-byte aligned and its valid part is whole float4s
            if ((O & 3) == 0 && (reinterpret_cast<uintptr_t>(direct) & 15) == 0) {
                for (int e = t * 4; e < BIC * BN * K; e += MFMA_THREADS * 4) {
                    const int il = e / (BN * K), rem = e % (BN * K);
                    if (i0 + il < I && rem < cols_here * K)
                        *reinterpret_cast<floatx4*>(direct + ((int64_t)(i0 + il) * O + o0) * K + rem) =
                            *reinterpret_cast<const floatx4*>(lds + il * BN * K + rem);
                }
                copied = true;
            }
        }
        if constexpr (KP != K) {
            // even K: the LDS rows are padded, so four elements are gathered; the store is still one float4
            if ((O & 3) == 0 && (reinterpret_cast<uintptr_t>(direct) & 15) == 0) {
                for (int e = t * 4; e < BIC * BN * K; e += MFMA_THREADS * 4) {
                    const int il = e / (BN * K), rem = e % (BN * K);
                    if (i0 + il < I && rem < cols_here * K) {
                        floatx4 v;
#pragma unroll
                        for (int q = 0; q < 4; ++q) v[q] = lds[(il * BN + (rem + q) / K) * KP + (rem + q) % K];
                        *reinterpret_cast<floatx4*>(direct + ((int64_t)(i0 + il) * O + o0) * K + rem) = v;
                    }
                }
                copied = true;
            }
        }
        if (!copied) {
            for (int e = t; e < BIC * BN * K; e += MFMA_THREADS) {
                const int il = e / (BN * K), rem = e % (BN * K);
                const int col = rem / K, k = rem % K;
                if (i0 + il < I && col < cols_here)
                    direct[((int64_t)(i0 + il) * O + o0) * K + rem] = lds[(il * BN + col) * KP + k];
            }
        }
        CHEBYKAN_PROBE(3);
        return;
    }
    float* out = partial + (int64_t)slice * IK * O;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const floatx16 v = total[i][j] + acc[i][j];
            const int col = o0 + wn * WN + j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ml = wm * 64 + i * 32 + mfma_row(r, h);
                const int64_t mg = (int64_t)i0 * K + ml;
                if (ml < Cfg::BMR && mg < IK && col < O) out[mg * O + col] = v[r];
            }
        }
    CHEBYKAN_PROBE(3);
}

template <class Cfg, class Basis = ExactBasis>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
dC_mfma_kernel(const float* __restrict__ x, const float* __restrict__ dy, float* __restrict__ partial,
               int B, int I, int O, int n_tiles_o, int o_begin, int n_tiles_i, int n_slices, int rows_per_slice,
               typename Basis::Args bargs, float* __restrict__ direct)
{
    dC_mfma_body<Cfg, Basis>(x, dy, partial, B, I, O, n_tiles_o, o_begin, n_tiles_i, n_slices, rows_per_slice, bargs, direct,
                             (int)blockIdx.x);
}

// dC[i,o,k] = sum_s partial[s][(i,k)][o] in a fixed order: G slice groups take every G-th
// slice each, then the G group sums are added in group order.  Also turns the [(i,k)][o]
// rows of the partials into the caller's [i][o][k] layout through LDS, so that reads and
// writes are both unit-stride.  block = G slice groups x 32 outputs; grid = (ceil(O/32), I).
// G = 32 (1024 threads) shortens the serial chain per thread when there are many slices.
// Only the first o_count columns are summed and written (the rest of a row may belong to a tail
// that other kernels produce).  Dynamic LDS: G * 32 * ((D+1)|1) floats.
template <int D, int G>
__device__ __forceinline__ void dC_combine_body(const float* __restrict__ partial, float* __restrict__ dC, int I, int O,
                                                int o_count, int n_slices, int block_x, int block_y, float* lds)
{
    constexpr int K = D + 1, KP = K | 1;
    const int t = threadIdx.x;
    const int ol = t & 31, sg = t >> 5;
    const int oc = block_x * 32;
    const int i = block_y;
    const int o = oc + ol;
    const int64_t IK = (int64_t)I * K;
    const int64_t slice_stride = IK * O;
    float v[K];
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] = 0.0f;
    if (o < o_count) {
        const float* p = partial + (int64_t)sg * slice_stride + (int64_t)i * K * O + o;
        int s = sg;
        // two slices per trip: both sets of loads are issued before either is added
        for (; s + G < n_slices; s += 2 * G, p += 2 * G * slice_stride) {
            float a[K], b[K];
#pragma unroll
            for (int k = 0; k < K; ++k) { a[k] = p[(int64_t)k * O]; b[k] = p[G * slice_stride + (int64_t)k * O]; }
#pragma unroll
            for (int k = 0; k < K; ++k) { v[k] += a[k]; v[k] += b[k]; }
        }
        if (s < n_slices) {
#pragma unroll
            for (int k = 0; k < K; ++k) v[k] += p[(int64_t)k * O];
        }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) lds[(sg * 32 + ol) * KP + k] = v[k];
    __syncthreads();
    const int n_valid = (o_count - oc < 32 ? o_count - oc : 32) * K;
    float* dst = dC + ((int64_t)i * O + oc) * K;
    for (int e = t; e < n_valid; e += G * 32) {
        const int o2 = e / K, k = e % K;
        float total = 0.0f;
#pragma unroll
        for (int q = 0; q < G; ++q) total += lds[(q * 32 + o2) * KP + k];
        dst[e] = total;
    }
}

template <int D, int G>
__global__ void __launch_bounds__(G * 32)
dC_combine_kernel(const float* __restrict__ partial, float* __restrict__ dC, int I, int O, int o_count, int n_slices)
{
    extern __shared__ __align__(16) float lds[];
    dC_combine_body<D, G>(partial, dC, I, O, o_count, n_slices, blockIdx.x, blockIdx.y, lds);
}

// Every slice sum of a stack's backward pass in ONE launch (the per-layer sums are tiny,
// latency-bound kernels: three launches of ~5 us each for the tabular stack).  A job is one
// layer's sum; kind 0 is dC_combine_kernel's [slice][(i,k)][o] -> [i][o][k], kind 1 a plain
// sum of [slice][n] planes (narrow layers).  1024 threads, 32 slice groups in both kinds.
struct CombineJob {
    const float* partial;
    float* out;
    int I, O, slices, kind;
    int64_t n;            // kind 1: elements per plane
    int first_block;      // filled in by the launcher
};
constexpr int COMBINE_MAX_JOBS = 8;
struct CombineArgs {
    CombineJob job[COMBINE_MAX_JOBS];
    int n_jobs;
};
inline int combine_job_blocks(const CombineJob& j)
{
    return j.kind == 0 ? ((j.O + 31) / 32) * j.I : (int)((j.n + 31) / 32);
}

template <int D>
__global__ void __launch_bounds__(1024) stack_combine_kernel(CombineArgs a)
{
    extern __shared__ __align__(16) float lds[];
    int q = 0;
    while (q + 1 < a.n_jobs && (int)blockIdx.x >= a.job[q + 1].first_block) ++q;
    const CombineJob& j = a.job[q];
    const int b = blockIdx.x - j.first_block;
    if (j.kind == 0) {
        const int gx = (j.O + 31) / 32;
        dC_combine_body<D, 32>(j.partial, j.out, j.I, j.O, j.O, j.slices, b % gx, b / gx, lds);
    } else {
        // 32 slice groups x 32 elements; groups add every 32nd slice, then the group sums in order
        const int el = threadIdx.x & 31, sg = threadIdx.x >> 5;
        const int64_t e = (int64_t)b * 32 + el;
        float s = 0.0f;
        if (e < j.n)
            for (int sl = sg; sl < j.slices; sl += 32) s += j.partial[(int64_t)sl * j.n + e];
        lds[sg * 33 + el] = s;
        __syncthreads();
        if (sg == 0 && e < j.n) {
            float total = 0.0f;
#pragma unroll
            for (int g = 0; g < 32; ++g) total += lds[g * 33 + el];
            j.out[e] = total;
        }
    }
}

// ============================================================ input gradient
// RB_ = 32-row blocks of the tile that can hold real rows.  4: wave w takes row block w and all
// NB column blocks.  1 or 2 (a batch of at most 32 or 64 rows): wave w takes column block w and
// the RB row blocks, so no MFMA is issued for row blocks that are all padding.
template <int D_, int NB_, int VEC_, int RB_ = 4>
struct DxCfg {
    static constexpr int D = D_, K = D_ + 1, NB = NB_, VEC = VEC_, RB = RB_;
    static constexpr int NACC = RB == 4 ? NB : RB;      // accumulators per wave
    static_assert(RB == 4 || RB == 1 || RB == 2, "row blocks");
    static constexpr int BM = 128;
    static constexpr int BNC = 32 * NB;                 // tile columns (NB MFMA column blocks)
    static constexpr int BIX = BNC / D;                 // input features per tile
    static constexpr int BNR = BIX * D;                 // real columns (i, k=1..D)
    static constexpr int BO = 32;                       // outputs per contraction chunk
    static constexpr int SAX = BO + 4;                  // row stride of the dy tile: 16-byte aligned rows, stride/4 odd
    static constexpr int SSX = BO * K + (D % 32);       // slab stride = D (mod 32): column n hits bank n
    static constexpr int A_FLOATS = (BM * SAX + 3) & ~3;
    static constexpr int B_FLOATS = (BIX * SSX + 3) & ~3;
    static constexpr int STAGE = A_FLOATS + B_FLOATS;
    static constexpr int SG = BNC + 1;                  // row stride of the G tile in the epilogue
    static constexpr int LDS_FLOATS = (2 * STAGE > BM * SG) ? 2 * STAGE : BM * SG;
    static constexpr int LDS_BYTES = LDS_FLOATS * 4;
    static constexpr int NSTEP = BO / 2;
    static constexpr int FOLD = FOLD_TERMS / BO;
    static constexpr int NEA = BM * BO;
    static constexpr int APT = NEA / VEC / MFMA_THREADS;
    static constexpr int NEB = BIX * BO * K;
    static constexpr int CPT = (NEB / VEC + MFMA_THREADS - 1) / MFMA_THREADS;
    static constexpr int EPT = (BM * BIX + MFMA_THREADS - 1) / MFMA_THREADS;
    static_assert(D >= 1 && BIX >= 1, "degree 0 has no input gradient");
    static_assert(VEC == 4, "tiles are copied 16 bytes at a time");
    static_assert((BO * K) % VEC == 0 && NEA % (VEC * MFMA_THREADS) == 0 && NSTEP % 4 == 0, "vector width");
};

// dx[b,i] = (1-u^2) sum_o dy[b,o] sum_{k>=1} C[i,o,k] T_k'(u),  u = tanh x[b,i]
// (paper Alg. 2, x_grad, with the chain rule through tanh).  The sum over o runs on the
// matrix cores as G = dy * W^T; the sum over k is the epilogue.  No atomics: one
// workgroup owns all outputs o for its (b,i) tile.  Each of the four waves takes 32 rows
// and all NB column blocks; NB is chosen on the host so that the feature count wastes
// as few columns as possible.  grid.x = ceil(B/128) * ceil(I/BIX).
template <class Cfg, class Basis = ExactBasis>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
dx_mfma_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
               float* __restrict__ dx, int B, int I, int O, int n_tiles_i, int chunks_per_split, int i_begin,
               typename Basis::Args bargs)
{
    constexpr int D = Cfg::D, K = Cfg::K, VEC = Cfg::VEC, BIX = Cfg::BIX, BO = Cfg::BO, NB = Cfg::NB;
    constexpr int SAX = Cfg::SAX, SSX = Cfg::SSX, SG = Cfg::SG;
    extern __shared__ __align__(16) float lds[];
    CHEBYKAN_PROBE(0);
    const Basis basis(bargs, lds + Cfg::LDS_BYTES / 4, Cfg::K, (int)threadIdx.x, MFMA_THREADS);

    const int t = threadIdx.x;
    const int tile_i = blockIdx.x % n_tiles_i;
    const int tile_b = blockIdx.x / n_tiles_i;
    const int b0 = tile_b * Cfg::BM;
    const int i0 = i_begin + tile_i * BIX;   // the launch covers the features from i_begin on

    // Views based at this tile.  Rows past B and features past I read as zero.  Outputs past O
    // (last chunk only) would read the next dy row / the next feature's slab: the dy value is
    // replaced by zero there, which removes the term whatever the coefficient operand holds.
    const int rows_here = B - b0 < Cfg::BM ? B - b0 : Cfg::BM;
    const BufferView gv = make_view(dy + (int64_t)b0 * O, (int64_t)rows_here * O);
    const BufferView cv = make_view(C + (int64_t)i0 * O * K, (int64_t)(I - i0) * O * K);
    const uint32_t OK_ = (uint32_t)O * (uint32_t)K;

    bufx4 areg[Cfg::APT];
    bufx4 creg[Cfg::CPT];
    // coefficient element handled in round j; past-the-end threads repeat the last vector
    int ce[Cfg::CPT];
#pragma unroll
    for (int j = 0; j < Cfg::CPT; ++j) {
        const int e = (t + j * MFMA_THREADS) * VEC;
        ce[j] = e < Cfg::NEB ? e : Cfg::NEB - VEC;
    }

    // Producer work of a chunk as a list of items: the LDS writes of chunk c+1 (dy vectors, then
    // coefficient vectors; held in registers since the previous iteration), then the global loads of
    // chunk c+2 into the same registers.  ragged = true only for the chunk that holds the end of the
    // dy rows: a vector may run past the end of its row there, element by element.
    constexpr int APT = Cfg::APT, CPT = Cfg::CPT, NITEM = 2 * (APT + CPT);
    auto item = [&](float* sA, float* sB, int oc, int q, auto ragged) {
        if (q < APT) {
            const int e = (t + q * MFMA_THREADS) * VEC;
            const floatx4 v = {areg[q][0], areg[q][1], areg[q][2], areg[q][3]};
            *reinterpret_cast<floatx4*>(sA + (e / BO) * SAX + e % BO) = v;
        } else if (q < APT + CPT) {
            const int j = q - APT;
            const int il = ce[j] / (BO * K), rem = ce[j] % (BO * K);
            if constexpr (SSX % 4 == 0) {
                const floatx4 v = {creg[j][0], creg[j][1], creg[j][2], creg[j][3]};
                *reinterpret_cast<floatx4*>(sB + il * SSX + rem) = v;
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) sB[il * SSX + rem + v] = creg[j][v];
            }
        } else if (q < 2 * APT + CPT) {
            const int j = q - APT - CPT;
            const int e = (t + j * MFMA_THREADS) * VEC;
            const int m = e / BO, kk = e % BO;
            // any 4-byte aligned position
            const bufx4 v = load4(gv, (uint32_t)m * (uint32_t)O + (uint32_t)(oc + kk));
            if constexpr (decltype(ragged)::value) {
#pragma unroll
                for (int w = 0; w < 4; ++w) areg[j][w] = oc + kk + w < O ? v[w] : 0.0f;
            } else {
                areg[j] = v;
            }
        } else {
            const int j = q - 2 * APT - CPT;
            const int il = ce[j] / (BO * K), rem = ce[j] % (BO * K);
            creg[j] = load4(cv, (uint32_t)il * OK_ + (uint32_t)oc * (uint32_t)K + (uint32_t)rem);
        }
    };
    using Plain = std::false_type;
    using Ragged = std::true_type;
    auto load_chunk = [&](int oc) {
#pragma unroll
        for (int q = APT + CPT; q < NITEM; ++q) item(nullptr, nullptr, oc, q, Ragged{});
    };
    auto store_chunk = [&](float* sA, float* sB) {
#pragma unroll
        for (int q = 0; q < APT + CPT; ++q) item(sA, sB, 0, q, Plain{});
    };

    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int aBase = (wave * 32 + l32) * SAX + h * (BO / 2);
    int bBase[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int n = j * 32 + l32;
        int il = n / D;
        const int kq = n % D;
        if (il > BIX - 1) il = BIX - 1;            // padding columns read valid memory, result unused
        bBase[j] = il * SSX + h * (BO / 2) * K + kq + 1;
    }

    constexpr int NACC = Cfg::NACC;
    floatx16 acc[NACC], total[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) { acc[j] = zero16(); total[j] = zero16(); }
    // small batch: this wave's column block (a wave beyond the last block repeats it and stores nothing)
    const int my_block = wave < NB ? wave : NB - 1;
    int bBaseSmall = bBase[0];
#pragma unroll
    for (int j = 1; j < NB; ++j) bBaseSmall = my_block == j ? bBase[j] : bBaseSmall;
    const int aBaseSmall = l32 * SAX + h * (BO / 2);

    // Operands.  A lane's dy values of consecutive steps are consecutive in its tile row: four steps
    // (a group) per 16-byte read, the next group fetched while this one is used.  Its coefficients lie
    // K words apart: single reads at immediate offsets (see lds_operand), LA steps ahead.
    constexpr int NSTEP = Cfg::NSTEP, NGROUP = NSTEP / 4, LA = LOOKAHEAD;
    constexpr int NAQ = Cfg::RB == 4 ? 1 : NACC;        // dy rows per lane
    constexpr int NBQ = Cfg::RB == 4 ? NB : 1;          // coefficient columns per lane
    floatx4 aq[NAQ][2];
    float bq[NSTEP][NBQ];
    auto read_a = [&](const float* sA, int g) {
#pragma unroll
        for (int i = 0; i < NAQ; ++i)
            aq[i][g & 1] = *reinterpret_cast<const floatx4*>(sA + (Cfg::RB == 4 ? aBase : aBaseSmall + i * 32 * SAX) + 4 * g);
    };
    auto read_b = [&](const float* sB, int s) {
#pragma unroll
        for (int j = 0; j < NBQ; ++j) bq[s][j] = lds_operand(sB + (Cfg::RB == 4 ? bBase[j] : bBaseSmall) + s * K);
    };

    // chunks past the last one are loaded and stored too (all-zero dy, stage never read).
    // blockIdx.y selects a range of chunks: the epilogue is linear in the accumulators, so a split
    // contraction writes partial dx planes that a second kernel adds in range order.
    const int n_chunks_all = (O + BO - 1) / BO;
    const int c_begin = blockIdx.y * chunks_per_split;
    const int n_chunks = n_chunks_all - c_begin < chunks_per_split ? n_chunks_all - c_begin : chunks_per_split;
    dx += (int64_t)blockIdx.y * B * I;

    // One chunk; the instruction order is laid down by hand, one step (NACC independent MFMAs) at a
    // time with a scheduling fence after each.
    auto chunk_body = [&](int c, auto ragged) {
        __syncthreads();   // stage c is complete; every wave has finished reading stage c+1
        const float* sA = lds + (c & 1) * Cfg::STAGE;
        const float* sB = sA + Cfg::A_FLOATS;
        float* nA = lds + ((c + 1) & 1) * Cfg::STAGE;
        float* nB = nA + Cfg::A_FLOATS;
        const int oc_next = (c_begin + c + 2) * BO;
        read_a(sA, 0);
#pragma unroll
        for (int s = 0; s < LA; ++s) read_b(sB, s);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            const int g = s / 4, m = s % 4;
            if (m == 1 && g + 1 < NGROUP) read_a(sA, g + 1);
            if (s + LA < NSTEP) read_b(sB, s + LA);
#pragma unroll
            for (int q = 0; q < NITEM; ++q)
                if (q * NSTEP / NITEM == s) item(nA, nB, oc_next, item_at(q, NITEM), ragged);
            if constexpr (Cfg::RB == 4) {
#pragma unroll
                for (int j = 0; j < NB; ++j) acc[j] = mfma32(aq[0][g & 1][m], bq[s][j], acc[j]);
            } else {
#pragma unroll
                for (int i = 0; i < NACC; ++i) acc[i] = mfma32(aq[i][g & 1][m], bq[s][0], acc[i]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    load_chunk(c_begin * BO);
    store_chunk(lds, lds + Cfg::A_FLOATS);
    load_chunk((c_begin + 1) * BO);
    // blocks of FOLD chunks, each closed by a fold of the accumulators
    for (int cf = 0; cf < n_chunks; cf += Cfg::FOLD) {
        const int c_end = cf + Cfg::FOLD < n_chunks ? cf + Cfg::FOLD : n_chunks;
        // chunk c+2 is loaded in iteration c: plain while that chunk ends inside the rows (chunks that
        // begin past the row end hold nothing that is read)
        const int c_plain = O / BO - 2 - c_begin < c_end ? O / BO - 2 - c_begin : c_end;
        int c = cf;
        for (; c < c_plain; ++c) chunk_body(c, Plain{});
        for (; c < c_end; ++c) chunk_body(c, Ragged{});
#pragma unroll
        for (int j = 0; j < NACC; ++j) { total[j] += acc[j]; acc[j] = zero16(); }
    }

    // --- epilogue: G tile to LDS, then each thread finishes (row, feature) pairs
    __syncthreads();
    if constexpr (Cfg::RB == 4) {
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const floatx16 v = total[j] + acc[j];
            const int col = j * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) lds[(wave * 32 + mfma_row(r, h)) * SG + col] = v[r];
        }
    } else if (wave < NB) {   // rows past 32 * RB of the G tile are not written and not read (they are past B)
#pragma unroll
        for (int i = 0; i < NACC; ++i) {
            const floatx16 v = total[i] + acc[i];
            const int col = wave * 32 + l32;
#pragma unroll
            for (int r = 0; r < 16; ++r) lds[(i * 32 + mfma_row(r, h)) * SG + col] = v[r];
        }
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < Cfg::EPT; ++j) {
        const int e = t + j * MFMA_THREADS;
        const int m = e / BIX, il = e % BIX;
        const int b = b0 + m, i = i0 + il;
        if (e < Cfg::BM * BIX && b < B && i < I) {
            float slope;
            float dT[D];
            basis.template dT<D>(x[(int64_t)b * I + i], dT, slope);
            const float* g = lds + m * SG + il * D;
            float sum = 0.0f;
#pragma unroll
            for (int k = 0; k < D; ++k) sum = fmaf(g[k], dT[k], sum);
            dx[(int64_t)b * I + i] = slope * sum;
        }
    }
}

// ------------------------------------------------ input gradient, feature-per-lane form
// Same operation as dx_mfma_kernel, other column order: a tile is 128 rows x 32 input
// features, and column block j of G holds degree k = j+1 for those 32 features.  The D
// accumulators of one lane then all belong to the SAME (row, feature) pairs, so the sum over
// k with T_k'(u) is taken in registers: no LDS round trip, no shuffles, and x / dx are
// accessed with consecutive lanes on consecutive features.  Because that sum is linear in the
// accumulators it is also what folds long contractions: every 512 outputs the accumulators
// are folded into 16 running dx values per lane.  Used whenever the feature count fills the
// 32-feature tiles reasonably; very narrow inputs stay with dx_mfma_kernel.
//
// The contraction index of this product (the output o) is the fast index of both operands as
// they lie in HBM: of a dy row, and - together with k - of a feature's coefficient run
// C[i][o][0..K).  Both tiles are therefore copied verbatim, 16 bytes at a time, into LDS rows
//     sA[row][BO (+4)]      sB[feature][BO*K (+4)]
// and a lane fetches the operands of four contraction steps with 16-byte LDS reads at immediate
// offsets from one base: one read of its dy row and K reads of its feature's run, for 4*D MFMAs.
// Row strides are 16-byte aligned with stride/4 odd, so that consecutive lanes' 16-byte accesses
// fall on distinct banks.  The k = 0 coefficients travel with the rest and are not used.
template <int D_, int VEC_>
struct Dx2Cfg {
    static constexpr int D = D_, K = D_ + 1, VEC = VEC_;
    static constexpr int BM = 128, BF = 32;
    static constexpr int BO = D <= 4 ? 32 : 16;         // outputs per contraction chunk
    static constexpr int SAX = BO + 4;                  // row stride of the dy tile
    static constexpr int SSX = BO * K + 4;              // stride of a feature's coefficient run
    static constexpr int A_FLOATS = BM * SAX;
    static constexpr int B_FLOATS = BF * SSX;
    static constexpr int STAGE = A_FLOATS + B_FLOATS;
    static constexpr int LDS_BYTES = 2 * STAGE * 4;
    static constexpr int NSTEP = BO / 2;                // MFMA steps per chunk: a step takes one output from each lane half
    static constexpr int NGROUP = NSTEP / 4;            // operand fetches per chunk: four steps each
    static constexpr int FOLD = FOLD_TERMS / BO;
    // producers: two threads per dy row, eight threads per feature run; every address is a
    // per-thread base plus a compile-time offset
    static constexpr int A_PER = BO / 2;                // dy floats per thread and chunk
    static constexpr int A_NV = A_PER / 4;
    static constexpr int RUN = BO * K;                  // floats of one feature's coefficient run
    static constexpr int C_PER = RUN / 8;               // per thread
    static constexpr int C_NV = C_PER / 4;              // full vectors per thread
    static constexpr int C_NS = C_PER - C_NV * 4;       // single floats per thread
    static_assert(D >= 1, "degree 0 has no input gradient");
    static_assert(VEC == 4, "tiles are copied 16 bytes at a time");
    static_assert(A_PER % 4 == 0 && RUN % 8 == 0 && NSTEP % 4 == 0, "split");
    static_assert((SAX / 4) % 2 == 1 && (SSX / 4) % 2 == 1 && SAX % 4 == 0 && SSX % 4 == 0, "bank spread of 16-byte rows");
};

// grid.x = ceil(B/128) * n_tiles_i, feature tile fastest.  The launch covers features [0, i_count)
// (all I of them, or the full tiles when a second launch takes the remainder).
template <class Cfg, class Basis = ExactBasis>
__global__ void __launch_bounds__(MFMA_THREADS, 2)
dx2_mfma_kernel(const float* __restrict__ x, const float* __restrict__ C, const float* __restrict__ dy,
                float* __restrict__ dx, int B, int I, int O, int n_tiles_i, int chunks_per_split, int i_count,
                typename Basis::Args bargs)
{
    constexpr int D = Cfg::D, K = Cfg::K, BF = Cfg::BF, BO = Cfg::BO;
    constexpr int SAX = Cfg::SAX, SSX = Cfg::SSX, NSTEP = Cfg::NSTEP, NGROUP = Cfg::NGROUP;
    extern __shared__ __align__(16) float lds[];
    CHEBYKAN_PROBE(0);
    const Basis basis(bargs, lds + Cfg::LDS_BYTES / 4, Cfg::K, (int)threadIdx.x, MFMA_THREADS);

    const int t = threadIdx.x;
    const int tile_i = blockIdx.x % n_tiles_i;
    const int tile_b = blockIdx.x / n_tiles_i;
    const int b0 = tile_b * Cfg::BM;
    const int i0 = tile_i * BF;
    const int lane = t & 63, wave = t >> 6;
    const int l32 = lane & 31, h = lane >> 5;

    // Views based at this tile: rows past B and features past I read as zero; outputs past O
    // (last chunk) are removed by zeroing the dy operand.
    const int rows_here = B - b0 < Cfg::BM ? B - b0 : Cfg::BM;
    const BufferView gv = make_view(dy + (int64_t)b0 * O, (int64_t)rows_here * O);
    const BufferView cv = make_view(C + (int64_t)i0 * O * K, (int64_t)(I - i0) * O * K);
    const BufferView xv = make_view(x + (int64_t)b0 * I, (int64_t)rows_here * I);
    const uint32_t OK_ = (uint32_t)O * (uint32_t)K;

    // this lane's 16 (row, feature) pairs: requested now, used in the epilogue
    const bool f_ok = i0 + l32 < i_count;
    float xval[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float v = load1(xv, (uint32_t)(wave * 32 + mfma_row(r, h)) * (uint32_t)I + (uint32_t)(i0 + l32));
        xval[r] = f_ok ? v : 0.0f;
    }

    bufx4 areg[Cfg::A_NV];
    bufx4 creg[Cfg::C_NV > 0 ? Cfg::C_NV : 1];
    float cone[Cfg::C_NS > 0 ? Cfg::C_NS : 1];
    const int pa_row = t >> 1, pa_part = t & 1;        // dy tile: row and half-row of this thread
    const int pc_f = t >> 3, pc_part = t & 7;          // coefficient run: feature and eighth
    const uint32_t ga_off = (uint32_t)pa_row * (uint32_t)O + (uint32_t)(pa_part * 4);
    const uint32_t gc_off = (uint32_t)pc_f * OK_;
    const int la_off = pa_row * SAX + pa_part * 4;
    const int lc_off = pc_f * SSX;

    // ragged = true (below) only for the chunk that holds the end of the dy rows: a vector may run
    // past the end of its row there, element by element
    const int aBase = (wave * 32 + l32) * SAX + h * NSTEP;
    const int bBase = l32 * SSX + h * NSTEP * K;

    floatx16 acc[D];
#pragma unroll
    for (int j = 0; j < D; ++j) acc[j] = zero16();
    float dxacc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) dxacc[r] = 0.0f;

    // dxacc += (1-u^2) sum_k acc_k T_k'(u), then acc = 0.  The empty asm makes x opaque here: the
    // derivative values of the 16 rows are recomputed at every fold instead of living in 16 x (D+1)
    // registers across the chunk loop, where the compiler would otherwise keep them.
    auto fold = [&]() {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float xr = xval[r];
            CHEBYKAN_OPAQUE(xr);
            float slope;
            float dT[D];
            basis.template dT<D>(xr, dT, slope);
            float sum = 0.0f;
#pragma unroll
            for (int j = 0; j < D; ++j) sum = fmaf(acc[j][r], dT[j], sum);
            dxacc[r] = fmaf(slope, sum, dxacc[r]);
        }
#pragma unroll
        for (int j = 0; j < D; ++j) acc[j] = zero16();
    };

    // Operands of four steps (a group): 4 dy values and the 4 x K coefficients of this lane's feature,
    // K + 1 reads of 16 bytes.  Item i of a group is its i-th read (0: dy, 1..K: coefficients).
    floatx4 aop[2], bop[2][K];
    auto read_item = [&](const float* sA, const float* sB, int g, int i) {
        if (i == 0) aop[g & 1] = *reinterpret_cast<const floatx4*>(sA + aBase + 4 * g);
        else bop[g & 1][i - 1] = *reinterpret_cast<const floatx4*>(sB + bBase + 4 * g * K + 4 * (i - 1));
    };
    // Producer work of a chunk as a list of items: first the LDS writes of chunk c+1 (held in registers
    // since the previous iteration), then the global loads of chunk c+2 into the same registers.
    constexpr int NW = Cfg::A_NV + Cfg::C_NV + Cfg::C_NS;
    auto store_item = [&](float* sA, float* sB, int i) {
        if (i < Cfg::A_NV) {
            const floatx4 v = {areg[i][0], areg[i][1], areg[i][2], areg[i][3]};
            *reinterpret_cast<floatx4*>(sA + la_off + i * 8) = v;
        } else if (i < Cfg::A_NV + Cfg::C_NV) {
            const int j = i - Cfg::A_NV;
            const floatx4 v = {creg[j][0], creg[j][1], creg[j][2], creg[j][3]};
            *reinterpret_cast<floatx4*>(sB + lc_off + pc_part * 4 + j * 32) = v;
        } else {
            const int j = i - Cfg::A_NV - Cfg::C_NV;
            sB[lc_off + Cfg::C_NV * 32 + pc_part + j * 8] = cone[j];
        }
    };
    auto load_item = [&](int oc, int i, auto ragged) {
        if (i < Cfg::A_NV) {
            const bufx4 v = load4(gv, ga_off + (uint32_t)(oc + i * 8));   // any 4-byte aligned position
            if constexpr (decltype(ragged)::value) {
                const int kk = oc + pa_part * 4 + i * 8;                  // first output of this vector
#pragma unroll
                for (int q = 0; q < 4; ++q) areg[i][q] = kk + q < O ? v[q] : 0.0f;
            } else {
                areg[i] = v;
            }
        } else if (i < Cfg::A_NV + Cfg::C_NV) {
            const int j = i - Cfg::A_NV;
            creg[j] = load4(cv, gc_off + (uint32_t)oc * (uint32_t)K + (uint32_t)(pc_part * 4 + j * 32));
        } else {
            const int j = i - Cfg::A_NV - Cfg::C_NV;
            cone[j] = load1(cv, gc_off + (uint32_t)oc * (uint32_t)K + (uint32_t)(Cfg::C_NV * 32 + pc_part + j * 8));
        }
    };
    auto load_chunk = [&](int oc, auto ragged) {
#pragma unroll
        for (int i = 0; i < NW; ++i) load_item(oc, i, ragged);
    };
    auto store_chunk = [&](float* sA, float* sB) {
#pragma unroll
        for (int i = 0; i < NW; ++i) store_item(sA, sB, i);
    };

    // chunks past the last one are loaded and stored too (all-zero dy, stage never read).
    // blockIdx.y selects a range of chunks: the epilogue is linear in the accumulators, so a split
    // contraction writes partial dx planes that a second kernel adds in range order.
    const int n_chunks_all = (O + BO - 1) / BO;
    const int c_begin = blockIdx.y * chunks_per_split;
    const int n_chunks = n_chunks_all - c_begin < chunks_per_split ? n_chunks_all - c_begin : chunks_per_split;
    dx += (int64_t)blockIdx.y * B * I;

    using Plain = std::false_type;
    using Ragged = std::true_type;
    // One chunk.  The instruction order is laid down by hand, one step (D independent MFMAs) at a
    // time with a scheduling fence after each: next to a step's MFMAs sit its share of the reads of
    // the next group, and its share of the producer items - none of them vector-ALU work, so
    // the matrix pipe is only ever interrupted by issue slots.
    auto chunk_body = [&](int c, auto ragged) {
        __syncthreads();   // stage c is complete; every wave has finished reading stage c+1
        const float* sA = lds + (c & 1) * Cfg::STAGE;
        const float* sB = sA + Cfg::A_FLOATS;
        float* nA = lds + ((c + 1) & 1) * Cfg::STAGE;
        float* nB = nA + Cfg::A_FLOATS;
        const int oc_next = (c_begin + c + 2) * BO;
#pragma unroll
        for (int i = 0; i <= K; ++i) read_item(sA, sB, 0, i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < NSTEP; ++s) {
            const int g = s / 4, m = s % 4;
            if (g + 1 < NGROUP) {
#pragma unroll
                for (int i = 0; i <= K; ++i)
                    if (i * 4 / (K + 1) == m) read_item(sA, sB, g + 1, i);
            }
#pragma unroll
            for (int i = 0; i < 2 * NW; ++i)
                if (i * NSTEP / (2 * NW) == s) {
                    if (i < NW) store_item(nA, nB, i);
                    else load_item(oc_next, i - NW, ragged);
                }
#pragma unroll
            for (int j = 0; j < D; ++j) {
                const int e = m * K + 1 + j;           // position in the group's run: step m, degree j+1
                acc[j] = mfma32(aop[g & 1][m], bop[g & 1][e / 4][e % 4], acc[j]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // the first two chunks of the range are loaded ahead of the loop; either may hold the row end
    if ((c_begin + 1) * BO <= O) load_chunk(c_begin * BO, Plain{}); else load_chunk(c_begin * BO, Ragged{});
    store_chunk(lds, lds + Cfg::A_FLOATS);
    if ((c_begin + 2) * BO <= O) load_chunk((c_begin + 1) * BO, Plain{}); else load_chunk((c_begin + 1) * BO, Ragged{});
    CHEBYKAN_PROBE(1);
    // blocks of FOLD chunks, each closed by a fold (the last one by the final fold)
    for (int cf = 0; cf < n_chunks; cf += Cfg::FOLD) {
        const int c_end = cf + Cfg::FOLD < n_chunks ? cf + Cfg::FOLD : n_chunks;
        // chunk c+2 is loaded in iteration c: plain while that chunk ends inside the rows (chunks that
        // begin past the row end hold nothing that is read)
        const int c_plain = O / BO - 2 - c_begin < c_end ? O / BO - 2 - c_begin : c_end;
        int c = cf;
        for (; c < c_plain; ++c) chunk_body(c, Plain{});
        for (; c < c_end; ++c) chunk_body(c, Ragged{});
        fold();
    }
    CHEBYKAN_PROBE(2);

    if (f_ok) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int row = b0 + wave * 32 + mfma_row(r, h);
            if (row < B) dx[(int64_t)row * I + i0 + l32] = dxacc[r];
        }
    }
    CHEBYKAN_PROBE(3);
}

}  // namespace chebykan
