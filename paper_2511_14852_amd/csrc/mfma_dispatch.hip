// Host side of the MFMA kernel family: which shapes it takes, tile choice,
// batch-slice plan for the coefficient gradient, launches.
#include <hip/hip_runtime.h>

#include "dispatch.h"
#include "mfma_kernels.h"

namespace chebykan {

namespace {

bool degree_specialised(int d) { return d == 3 || d == 4 || d == 5 || d == 6 || d == 8; }

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

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

// --------------------------------------------------------------------- dC
struct DcPlan {
    int bn;              // output tile width
    int slices;          // batch slices (partial buffers)
    int rows_per_slice;  // multiple of 32
};

DcPlan plan_dC(int64_t B, int I, int O, int d)
{
    const int K = d + 1;
    DcPlan p;
    p.bn = O <= 64 ? 64 : 128;
    const int bic = 128 / K;
    const int64_t tiles = (int64_t)((I + bic - 1) / bic) * ((O + p.bn - 1) / p.bn);
    int64_t want = (1024 + tiles - 1) / tiles;                 // aim for >= 1024 workgroups
    const int64_t max_by_rows = (B + 255) / 256;               // at least 256 rows per slice
    const int64_t bytes_per_slice = (int64_t)I * K * O * 4;
    const int64_t max_by_bytes = ((int64_t)512 << 20) / bytes_per_slice;
    if (want > max_by_rows) want = max_by_rows;
    if (want > max_by_bytes) want = max_by_bytes;
    if (want < 1) want = 1;
    int64_t rows = (B + want - 1) / want;
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
    hipLaunchKernelGGL(dC_mfma_kernel<Cfg>, dim3((unsigned)(tiles_i * tiles_o), (unsigned)p.slices),
                       dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, dy, partial, B, I, O, tiles_o, p.rows_per_slice);
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
    hipLaunchKernelGGL(dC_combine_kernel<D>, dim3((unsigned)((O + 255) / 256), (unsigned)I), dim3(256),
                       256 * ((D + 1) | 1) * sizeof(float), s, partial, dC, I, O, p.slices);
}

// --------------------------------------------------------------------- dx
template <int D, int VEC>
void launch_dx(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    using Cfg = DxCfg<D, VEC>;
    static bool once = (allow_lds(dx_mfma_kernel<Cfg>, Cfg::LDS_BYTES), true);
    (void)once;
    const int tiles_i = (I + Cfg::BIX - 1) / Cfg::BIX;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * tiles_i;
    hipLaunchKernelGGL(dx_mfma_kernel<Cfg>, dim3((unsigned)tiles), dim3(MFMA_THREADS), Cfg::LDS_BYTES, s, x, C, dy,
                       dx, B, I, O, tiles_i);
}

template <int D>
void pick_dx(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O, hipStream_t s)
{
    const bool vec = aligned16(C) && aligned16(dy) && O % 4 == 0;   // O%4==0 makes every slab run 16-byte aligned
    if (vec) launch_dx<D, 4>(x, C, dy, dx, B, I, O, s);
    else launch_dx<D, 1>(x, C, dy, dx, B, I, O, s);
}

bool shape_fits(int64_t B, int I, int O, int d)
{
    if (!degree_specialised(d)) return false;
    if (B > 0x7fffffff || I > 65535) return false;
    // grid.x limits: tiles stay below 2^31
    const int64_t tb = (B + 127) / 128;
    if (tb * ((O + 63) / 64) > 0x7fffffff || tb * I > 0x7fffffff) return false;
    return true;
}

}  // namespace

size_t forward_workspace_bytes(int64_t, int, int, int) { return 0; }

size_t backward_workspace_bytes(int64_t B, int I, int O, int d)
{
    if (B <= 0 || !shape_fits(B, I, O, d)) return 0;
    const DcPlan p = plan_dC(B, I, O, d);
    return (size_t)p.slices * (size_t)I * (size_t)(d + 1) * (size_t)O * sizeof(float);
}

bool mfma_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void*, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || O < 8) return false;   // very narrow outputs: not a matrix-core shape
    const int b = (int)B;
    switch (d) {
        case 3: pick_fwd<3, 8>(x, C, y, b, I, O, s); return true;
        case 4: pick_fwd<4, 8>(x, C, y, b, I, O, s); return true;
        case 5: pick_fwd<5, 6>(x, C, y, b, I, O, s); return true;
        case 6: pick_fwd<6, 4>(x, C, y, b, I, O, s); return true;
        case 8: pick_fwd<8, 4>(x, C, y, b, I, O, s); return true;
    }
    return false;
}

bool mfma_dx(const float* x, const float* C, const float* dy, float* dx, int64_t B, int I, int O, int d, void*,
             hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || O < 8) return false;
    const int b = (int)B;
    switch (d) {
        case 3: pick_dx<3>(x, C, dy, dx, b, I, O, s); return true;
        case 4: pick_dx<4>(x, C, dy, dx, b, I, O, s); return true;
        case 5: pick_dx<5>(x, C, dy, dx, b, I, O, s); return true;
        case 6: pick_dx<6>(x, C, dy, dx, b, I, O, s); return true;
        case 8: pick_dx<8>(x, C, dy, dx, b, I, O, s); return true;
    }
    return false;
}

bool mfma_dC(const float* x, const float* dy, float* dC, int64_t B, int I, int O, int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || O < 8 || !ws) return false;
    const DcPlan p = plan_dC(B, I, O, d);
    float* partial = static_cast<float*>(ws);
    const int b = (int)B;
    switch (d) {
        case 3: pick_dC<3>(x, dy, dC, partial, b, I, O, p, s); return true;
        case 4: pick_dC<4>(x, dy, dC, partial, b, I, O, p, s); return true;
        case 5: pick_dC<5>(x, dy, dC, partial, b, I, O, p, s); return true;
        case 6: pick_dC<6>(x, dy, dC, partial, b, I, O, p, s); return true;
        case 8: pick_dC<8>(x, dy, dC, partial, b, I, O, p, s); return true;
    }
    return false;
}

}  // namespace chebykan
