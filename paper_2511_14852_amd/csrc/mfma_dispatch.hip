// Host side of the MFMA kernel family: which shapes it takes, tile choice,
// batch-slice plan for the coefficient gradient, launches.
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "dispatch.h"
#include "mfma_kernels.h"
#include "narrow_kernels.h"

namespace chebykan {

namespace {

bool degree_specialised(int d) { return d == 3 || d == 4 || d == 5 || d == 6 || d == 8; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Tuning switches for kernel experiments: integer bit mask in the environment variable
// CHEBYKAN_TUNE, read once.  Bit 2 (value 4): always use the packed-column dx kernel.
int tune_flags()
{
    static const int flags = [] {
        const char* e = getenv("CHEBYKAN_TUNE");
        return e ? atoi(e) : 0;
    }();
    return flags;
}

// Dynamic LDS above 64 KiB has to be allowed per kernel once.
template <class KernelT>
void allow_lds(KernelT kernel, int bytes)
{
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                              bytes);
}

// ------------------------------------------------------------------ forward
template <int D, int BN, int BI, int VEC>
void launch_fwd(const float* x, const float* C, float* y, int B, int I, int O, hipStream_t s)
{
    using Cfg = FwdCfg<D, BN, BI, VEC>;
    static bool once = (allow_lds(fwd_mfma_kernel<Cfg>, Cfg::LDS_BYTES), true);
    (void)once;
    const int tiles_o = (O + BN - 1) / BN;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * tiles_o;
    hipLaunchKernelGGL(fwd_mfma_kernel<Cfg>, dim3((unsigned)tiles), dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, C,
                       y, B, I, O, tiles_o);
}

template <int D, int BI>
void pick_fwd(const float* x, const float* C, float* y, int B, int I, int O, hipStream_t s)
{
    const bool vec = aligned16(C) && ((int64_t)O * (D + 1)) % 4 == 0;
    if (O <= 64) {
        if (vec) launch_fwd<D, 64, BI, 4>(x, C, y, B, I, O, s);
        else launch_fwd<D, 64, BI, 1>(x, C, y, B, I, O, s);
    } else {
        if (vec) launch_fwd<D, 128, BI, 4>(x, C, y, B, I, O, s);
        else launch_fwd<D, 128, BI, 1>(x, C, y, B, I, O, s);
    }
}

bool use_narrow_shape(int I, int O, int d) { return O <= 4 && (int64_t)I * O * (d + 1) <= 16384; }

// --------------------------------------------------------------------- dC
struct DcPlan {
    int bn;              // output tile width
    int slices;          // batch slices (partial buffers)
    int rows_per_slice;  // multiple of 32
};

// Batch slices for the coefficient gradient.  512 workgroups are resident at once
// (256 CUs x 2); the slice count is the smallest one that fills at least one such
// round and wastes under a tenth of its last round, subject to >= 256 rows per slice
// and a 512 MiB cap on the partial buffers.
DcPlan plan_dC(int64_t B, int I, int O, int d)
{
    const int K = d + 1;
    DcPlan p;
    p.bn = O <= 64 ? 64 : 128;
    const int bic = 128 / K;
    const int64_t tiles = (int64_t)((I + bic - 1) / bic) * ((O + p.bn - 1) / p.bn);
    int64_t max_s = (B + 255) / 256;
    const int64_t bytes_per_slice = (int64_t)I * K * O * 4;
    const int64_t max_by_bytes = ((int64_t)512 << 20) / bytes_per_slice;
    if (max_s > max_by_bytes) max_s = max_by_bytes;
    if (max_s > 1024) max_s = 1024;
    if (max_s < 1) max_s = 1;
    int64_t best = 1;
    double best_eff = -1.0;
    for (int64_t sl = 1; sl <= max_s; ++sl) {
        const int64_t wg = tiles * sl;
        const int64_t rounds = (wg + 511) / 512;
        const double eff = (double)wg / (double)(rounds * 512);
        if (eff > best_eff + 1e-9) { best_eff = eff; best = sl; }
        if (wg >= 512 && eff >= 0.9) { best = sl; break; }
    }
    int64_t rows = (B + best - 1) / best;
    rows = (rows + 31) / 32 * 32;
    if (rows < 32) rows = 32;
    p.rows_per_slice = (int)rows;
    p.slices = (int)((B + rows - 1) / rows);
    if (p.slices < 1) p.slices = 1;
    return p;
}

template <int D, int BN, int VEC>
void launch_dC(const float* x, const float* dy, float* partial, int B, int I, int O, const DcPlan& p,
               hipStream_t s)
{
    using Cfg = DcCfg<D, BN, VEC>;
    static bool once = (allow_lds(dC_mfma_kernel<Cfg>, Cfg::LDS_BYTES), true);
    (void)once;
    const int tiles_o = (O + BN - 1) / BN;
    const int tiles_i = (I + Cfg::BIC - 1) / Cfg::BIC;
    hipLaunchKernelGGL(dC_mfma_kernel<Cfg>, dim3((unsigned)((int64_t)tiles_i * tiles_o * p.slices)),
                       dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, dy, partial, B, I, O, tiles_o, tiles_i, p.slices,
                       p.rows_per_slice);
}

template <int D>
void pick_dC(const float* x, const float* dy, float* dC, float* partial, int B, int I, int O, const DcPlan& p,
             hipStream_t s)
{
    const bool vec = aligned16(dy) && O % 4 == 0;
    if (p.bn == 64) {
        if (vec) launch_dC<D, 64, 4>(x, dy, partial, B, I, O, p, s);
        else launch_dC<D, 64, 1>(x, dy, partial, B, I, O, p, s);
    } else {
        if (vec) launch_dC<D, 128, 4>(x, dy, partial, B, I, O, p, s);
        else launch_dC<D, 128, 1>(x, dy, partial, B, I, O, p, s);
    }
    hipLaunchKernelGGL(dC_combine_kernel<D>, dim3((unsigned)((O + 31) / 32), (unsigned)I), dim3(256),
                       256 * ((D + 1) | 1) * sizeof(float), s, partial, dC, I, O, p.slices);
}

// --------------------------------------------------------------------- dx
template <int D, int NB, int VEC>
void launch_dx(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    using Cfg = DxCfg<D, NB, VEC>;
    static bool once = (allow_lds(dx_mfma_kernel<Cfg>, Cfg::LDS_BYTES), true);
    (void)once;
    const int tiles_i = (I + Cfg::BIX - 1) / Cfg::BIX;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * tiles_i;
    hipLaunchKernelGGL(dx_mfma_kernel<Cfg>, dim3((unsigned)tiles), dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, C, dy,
                       dx, B, I, O, tiles_i);
}

// Column blocks per tile: the count (1..4) that covers the I*D columns of G with the
// fewest 32-column MFMA blocks; ties go to the wider tile (more reuse of the dy tile).
int dx_column_blocks(int I, int D)
{
    int best = 4;
    int64_t best_cost = -1;
    for (int nb = 4; nb >= 1; --nb) {
        const int bix = 32 * nb / D;
        if (bix < 1) continue;
        const int64_t cost = (int64_t)((I + bix - 1) / bix) * nb;
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = nb; }
    }
    return best;
}

template <int D, int VEC>
void pick_dx_nb(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    switch (dx_column_blocks(I, D)) {
        case 1: launch_dx<D, 1, VEC>(x, C, dy, dx, B, I, O, s); break;
        case 2: launch_dx<D, 2, VEC>(x, C, dy, dx, B, I, O, s); break;
        case 3: launch_dx<D, 3, VEC>(x, C, dy, dx, B, I, O, s); break;
        default: launch_dx<D, 4, VEC>(x, C, dy, dx, B, I, O, s); break;
    }
}

template <int D, int VEC>
void launch_dx2(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    using Cfg = Dx2Cfg<D, VEC>;
    static bool once = (allow_lds(dx2_mfma_kernel<Cfg>, Cfg::LDS_BYTES), true);
    (void)once;
    const int tiles_i = (I + Cfg::BF - 1) / Cfg::BF;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * tiles_i;
    hipLaunchKernelGGL(dx2_mfma_kernel<Cfg>, dim3((unsigned)tiles), dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, C, dy,
                       dx, B, I, O, tiles_i);
}

// The feature-per-lane kernel works on 32-feature tiles; it is taken for degrees up to 6
// (measured slower at degree 8, where its eight accumulator blocks leave too few registers)
// unless it needs over 5 % more MFMA blocks than the packed-column kernel (ragged or very
// narrow feature counts).
bool dx_feature_per_lane(int I, int D)
{
    if (D > 6) return false;
    const int nb = dx_column_blocks(I, D);
    const int64_t packed = (int64_t)((I + 32 * nb / D - 1) / (32 * nb / D)) * nb;
    const int64_t per_lane = (int64_t)((I + 31) / 32) * D;
    return per_lane * 100 <= packed * 105;
}

template <int D>
void pick_dx(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    const bool vec = aligned16(C) && aligned16(dy) && O % 4 == 0;   // O%4==0 makes every slab run 16-byte aligned
    if (dx_feature_per_lane(I, D) && !(tune_flags() & 4)) {
        if (vec) launch_dx2<D, 4>(x, C, dy, dx, B, I, O, s);
        else launch_dx2<D, 1>(x, C, dy, dx, B, I, O, s);
    } else {
        if (vec) pick_dx_nb<D, 4>(x, C, dy, dx, B, I, O, s);
        else pick_dx_nb<D, 1>(x, C, dy, dx, B, I, O, s);
    }
}

bool shape_fits(int64_t B, int I, int O, int d)
{
    if (!degree_specialised(d)) return false;
    if (B > 0x7fffffff || I > 65535) return false;
    if ((int64_t)I * O * (d + 1) >= ((int64_t)1 << 30)) return false;   // 32-bit byte offsets into C
    // 32-bit byte offsets inside one batch slice of x and dy (a slice never exceeds B rows)
    if (B * (int64_t)(I > O ? I : O) >= ((int64_t)1 << 30) && !use_narrow_shape(I, O, d)) {
        const DcPlan p = plan_dC(B, I, O, d);
        if ((int64_t)p.rows_per_slice * (I > O ? I : O) >= ((int64_t)1 << 30)) return false;
    }
    // grid.x limits: tiles stay below 2^31
    const int64_t tb = (B + 127) / 128;
    if (tb * ((O + 63) / 64) > 0x7fffffff || tb * I > 0x7fffffff) return false;
    return true;
}

// ------------------------------------------------------------ narrow layers
constexpr int NARROW_MAX_OUT = 4;
constexpr int NARROW_FWD_WGS = 2048, NARROW_BWD_WGS = 512;

bool use_narrow(int64_t B, int I, int O, int d)
{
    return shape_fits(B, I, O, d) && O <= NARROW_MAX_OUT && (int64_t)I * O * (d + 1) <= 16384;
}

struct NarrowPlan {
    int G;             // lanes per row
    int rows_per_wg;   // multiple of NARROW_RB * (256 / G)
    int slices;        // workgroups along the batch
};

// `target`: workgroups to aim for (forward likes many short ones; backward pays for every
// slice again in the slice sum)
NarrowPlan plan_narrow(int64_t B, int I, int target)
{
    NarrowPlan p;
    p.G = 8;
    while (p.G < 64 && p.G < I) p.G *= 2;
    const int quantum = NARROW_RB * (NARROW_THREADS / p.G);
    int64_t rows = (B + target - 1) / target;
    rows = (rows + quantum - 1) / quantum * quantum;
    if (rows < quantum) rows = quantum;
    p.rows_per_wg = (int)rows;
    p.slices = (int)((B + rows - 1) / rows);
    if (p.slices < 1) p.slices = 1;
    return p;
}

template <int D, int O>
void launch_narrow_fwd(const float* x, const float* C, float* y, int B, int I, hipStream_t s)
{
    const NarrowPlan p = plan_narrow(B, I, NARROW_FWD_WGS);
    hipLaunchKernelGGL((narrow_fwd_kernel<D, O>), dim3((unsigned)p.slices), dim3(NARROW_THREADS),
                       (size_t)I * O * (D + 1) * sizeof(float), s, x, C, y, B, I, p.G, p.rows_per_wg);
}

template <int D, int O>
void launch_narrow_bwd(const float* x, const float* C, const float* dy, float* dx, float* dC, float* partial,
                       int B, int I, hipStream_t s)
{
    const NarrowPlan p = plan_narrow(B, I, NARROW_BWD_WGS);
    const int blocks_i = (I + p.G - 1) / p.G;
    hipLaunchKernelGGL((narrow_bwd_kernel<D, O>), dim3((unsigned)p.slices, (unsigned)blocks_i),
                       dim3(NARROW_THREADS), (size_t)NARROW_THREADS * O * (D + 1) * sizeof(float), s, x, C, dy,
                       dx, dC ? partial : nullptr, B, I, p.G, p.rows_per_wg);
    if (dC) {
        const int n = I * O * (D + 1);
        hipLaunchKernelGGL(sum_slices_kernel, dim3((unsigned)((n + 7) / 8)), dim3(256), 32 * 9 * sizeof(float), s,
                           partial, dC, n, p.slices);
    }
}

template <int D>
void narrow_fwd_by_out(const float* x, const float* C, float* y, int B, int I, int O, hipStream_t s)
{
    switch (O) {
        case 1: launch_narrow_fwd<D, 1>(x, C, y, B, I, s); break;
        case 2: launch_narrow_fwd<D, 2>(x, C, y, B, I, s); break;
        case 3: launch_narrow_fwd<D, 3>(x, C, y, B, I, s); break;
        default: launch_narrow_fwd<D, 4>(x, C, y, B, I, s); break;
    }
}

template <int D>
void narrow_bwd_by_out(const float* x, const float* C, const float* dy, float* dx, float* dC, float* partial, int B,
                       int I, int O, hipStream_t s)
{
    switch (O) {
        case 1: launch_narrow_bwd<D, 1>(x, C, dy, dx, dC, partial, B, I, s); break;
        case 2: launch_narrow_bwd<D, 2>(x, C, dy, dx, dC, partial, B, I, s); break;
        case 3: launch_narrow_bwd<D, 3>(x, C, dy, dx, dC, partial, B, I, s); break;
        default: launch_narrow_bwd<D, 4>(x, C, dy, dx, dC, partial, B, I, s); break;
    }
}

}  // namespace

size_t forward_workspace_bytes(int64_t, int, int, int) { return 0; }

size_t backward_workspace_bytes(int64_t B, int I, int O, int d)
{
    if (B <= 0 || !shape_fits(B, I, O, d)) return 0;
    const size_t coeffs = (size_t)I * (size_t)(d + 1) * (size_t)O * sizeof(float);
    if (use_narrow(B, I, O, d)) return (size_t)plan_narrow(B, I, NARROW_BWD_WGS).slices * coeffs;
    return (size_t)plan_dC(B, I, O, d).slices * coeffs;
}

bool fast_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void*, hipStream_t s)
{
    if (!shape_fits(B, I, O, d)) return false;
    const int b = (int)B;
    if (use_narrow(B, I, O, d)) {
        switch (d) {
            case 3: narrow_fwd_by_out<3>(x, C, y, b, I, O, s); return true;
            case 4: narrow_fwd_by_out<4>(x, C, y, b, I, O, s); return true;
            case 5: narrow_fwd_by_out<5>(x, C, y, b, I, O, s); return true;
            case 6: narrow_fwd_by_out<6>(x, C, y, b, I, O, s); return true;
            case 8: narrow_fwd_by_out<8>(x, C, y, b, I, O, s); return true;
        }
        return false;
    }
    switch (d) {
        case 3: pick_fwd<3, 8>(x, C, y, b, I, O, s); return true;
        case 4: pick_fwd<4, 8>(x, C, y, b, I, O, s); return true;
        case 5: pick_fwd<5, 6>(x, C, y, b, I, O, s); return true;
        case 6: pick_fwd<6, 4>(x, C, y, b, I, O, s); return true;
        case 8: pick_fwd<8, 4>(x, C, y, b, I, O, s); return true;
    }
    return false;
}

template <int D>
static void mfma_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, float* partial,
                          int B, int I, int O, hipStream_t s)
{
    if (dx) pick_dx<D>(x, C, dy, dx, B, I, O, s);
    if (dC) pick_dC<D>(x, dy, dC, partial, B, I, O, plan_dC(B, I, O, D), s);
}

bool fast_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int64_t B, int I, int O,
                   int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || (dC && !ws)) return false;
    float* partial = static_cast<float*>(ws);
    const int b = (int)B;
    if (use_narrow(B, I, O, d)) {
        switch (d) {
            case 3: narrow_bwd_by_out<3>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
            case 4: narrow_bwd_by_out<4>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
            case 5: narrow_bwd_by_out<5>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
            case 6: narrow_bwd_by_out<6>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
            case 8: narrow_bwd_by_out<8>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
        }
        return false;
    }
    switch (d) {
        case 3: mfma_backward<3>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
        case 4: mfma_backward<4>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
        case 5: mfma_backward<5>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
        case 6: mfma_backward<6>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
        case 8: mfma_backward<8>(x, C, dy, dx, dC, partial, b, I, O, s); return true;
    }
    return false;
}

}  // namespace chebykan
