// Host side of the specialised kernel families: workspace sizes and the switch from a
// runtime degree to the per-degree entry points (each compiled in its own deg_NN.hip).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "basis.h"
#include "chain_kernels.h"
#include "dispatch.h"
#include "launch.h"
#include "mfma_kernels.h"
#include "plans.h"

namespace chebykan {

template <int D, class Basis>
void degree_forward(const float* x, const float* C, float* y, int B, int I, int O, void* ws,
                    const typename Basis::Args& ba, hipStream_t s);
template <int D, class Basis>
void degree_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int B, int I, int O,
                     void* ws, const typename Basis::Args& ba, hipStream_t s);

#define CHEBYKAN_DECLARE_DEGREE(n)                                                                               \
    extern template void degree_forward<n, ExactBasis>(const float*, const float*, float*, int, int, int, void*,  \
                                                       const ExactBasis::Args&, hipStream_t);                     \
    extern template void degree_backward<n, ExactBasis>(const float*, const float*, const float*, float*, float*, \
                                                        int, int, int, void*, const ExactBasis::Args&, hipStream_t);
CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_DECLARE_DEGREE)
#undef CHEBYKAN_DECLARE_DEGREE
#define CHEBYKAN_DECLARE_TABLE_DEGREE(n)                                                                          \
    extern template void degree_forward<n, TableBasis>(const float*, const float*, float*, int, int, int, void*,  \
                                                       const TableBasis::Args&, hipStream_t);                     \
    extern template void degree_backward<n, TableBasis>(const float*, const float*, const float*, float*, float*, \
                                                        int, int, int, void*, const TableBasis::Args&, hipStream_t);
CHEBYKAN_FOR_EACH_TABLE_DEGREE(CHEBYKAN_DECLARE_TABLE_DEGREE)
#undef CHEBYKAN_DECLARE_TABLE_DEGREE
#define CHEBYKAN_DECLARE_DERIV_TABLE_DEGREE(n)                                                                          \
    extern template void degree_backward<n, DerivTableBasis>(const float*, const float*, const float*, float*, float*, \
                                                             int, int, int, void*, const DerivTableBasis::Args&, hipStream_t);
CHEBYKAN_FOR_EACH_TABLE_DEGREE(CHEBYKAN_DECLARE_DERIV_TABLE_DEGREE)
#undef CHEBYKAN_DECLARE_DERIV_TABLE_DEGREE

#define CHEBYKAN_DECLARE_FAMILY(n, Basis)                                                                      \
    extern template void degree_forward<n, Basis>(const float*, const float*, float*, int, int, int, void*,   \
                                                  const Basis::Args&, hipStream_t);                            \
    extern template void degree_backward<n, Basis>(const float*, const float*, const float*, float*, float*,  \
                                                   int, int, int, void*, const Basis::Args&, hipStream_t);
#define CHEBYKAN_DECLARE_POLY(n) CHEBYKAN_DECLARE_FAMILY(n, LegendreBasis) CHEBYKAN_DECLARE_FAMILY(n, HermiteBasis)
#define CHEBYKAN_DECLARE_FOURIER(n) CHEBYKAN_DECLARE_FAMILY(n, FourierBasis)
CHEBYKAN_FOR_EACH_FAMILY_DEGREE(CHEBYKAN_DECLARE_POLY)
CHEBYKAN_FOR_EACH_FOURIER_DEGREE(CHEBYKAN_DECLARE_FOURIER)
#undef CHEBYKAN_DECLARE_POLY
#undef CHEBYKAN_DECLARE_FOURIER
#undef CHEBYKAN_DECLARE_FAMILY

template <int D>
void degree_chain_forward(const ChainArgs& a, int B, hipStream_t s);
#define CHEBYKAN_DECLARE_CHAIN(n) extern template void degree_chain_forward<n>(const ChainArgs&, int, hipStream_t);
CHEBYKAN_FOR_EACH_CHAIN_DEGREE(CHEBYKAN_DECLARE_CHAIN)
#undef CHEBYKAN_DECLARE_CHAIN

thread_local CombineJob* g_deferred_combine = nullptr;

template <int D>
void degree_pair_backward(const PairArgs& a, CombineJob* jobs, hipStream_t s);
#define CHEBYKAN_DECLARE_PAIR(n) extern template void degree_pair_backward<n>(const PairArgs&, CombineJob*, hipStream_t);
CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_DECLARE_PAIR)
#undef CHEBYKAN_DECLARE_PAIR

template <int D>
void degree_stack_combine(CombineArgs& a, hipStream_t s);
#define CHEBYKAN_DECLARE_COMBINE(n) extern template void degree_stack_combine<n>(CombineArgs&, hipStream_t);
CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_DECLARE_COMBINE)
#undef CHEBYKAN_DECLARE_COMBINE

size_t forward_workspace_bytes(int64_t B, int I, int O, int d)
{
    if (B <= 0 || !shape_fits(B, I, O, d) || use_narrow(B, I, O, d)) return 0;
    const FwdPlan p = plan_forward(B, I, O, d);
    return p.splits > 1 ? (size_t)p.splits * (size_t)B * (size_t)O * sizeof(float) : 0;
}

size_t backward_workspace_bytes(int64_t B, int I, int O, int d)
{
    if (B <= 0 || !shape_fits(B, I, O, d)) return 0;
    const size_t coeffs = (size_t)I * (size_t)(d + 1) * (size_t)O * sizeof(float);
    if (use_narrow(B, I, O, d)) return (size_t)plan_narrow(B, I, NARROW_BWD_WGS).slices * coeffs;
    size_t for_dC = (size_t)plan_dC(B, I, O, d).slices * coeffs;
    const OutTiling ot = out_tiling(I, O, d);
    if (O > 64 && ot.tail_kind == 2)   // partials of the streamed tail columns lie behind those of the tiles
        for_dC += (size_t)plan_narrow(B, I, NARROW_BWD_WGS).slices * (size_t)I * (size_t)(O - ot.tail_begin) * (size_t)(d + 1) * sizeof(float);
    const DxPlan dxp = plan_dx(B, I, O, d);
    const size_t for_dx = dxp.split.splits > 1 ? (size_t)dxp.split.splits * (size_t)B * (size_t)I * sizeof(float) : 0;
    size_t need = for_dC > for_dx ? for_dC : for_dx;   // used one after the other on the same stream
    if (use_narrow_in(B, I, O, d)) {                     // the one-kernel path (both gradients requested)
        const size_t both = (size_t)plan_narrow_in(B).slices * coeffs;
        if (both > need) need = both;
    }
    return need;
}

bool fast_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d)) return false;
    if (forward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    switch (d) {
#define CHEBYKAN_FORWARD_CASE(n) case n: degree_forward<n, ExactBasis>(x, C, y, (int)B, I, O, ws, ExactBasis::Args{}, s); return true;
        CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_FORWARD_CASE)
#undef CHEBYKAN_FORWARD_CASE
    }
    return false;
}

bool fast_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int64_t B, int I, int O,
                   int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || (backward_workspace_bytes(B, I, O, d) > 0 && !ws)) return false;
    switch (d) {
#define CHEBYKAN_BACKWARD_CASE(n) case n: degree_backward<n, ExactBasis>(x, C, dy, dx, dC, (int)B, I, O, ws, ExactBasis::Args{}, s); return true;
        CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_BACKWARD_CASE)
#undef CHEBYKAN_BACKWARD_CASE
    }
    return false;
}

// ---- table-interpolated variant: same plans and workspace, basis read from an LDS copy of the table
bool table_fits(int d, int n)
{
    return table_degree_specialised(d) && n >= 2 && (int64_t)n * (d + 1) * (int64_t)sizeof(float) <= TABLE_LDS_BYTES;
}

bool fast_forward_table(const float* x, const float* C, const float* lut, int n, float* y, int64_t B, int I, int O,
                        int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || !table_fits(d, n)) return false;
    if (forward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    const TableBasis::Args ba{lut, n};
    switch (d) {
#define CHEBYKAN_FORWARD_CASE(k) case k: degree_forward<k, TableBasis>(x, C, y, (int)B, I, O, ws, ba, s); return true;
        CHEBYKAN_FOR_EACH_TABLE_DEGREE(CHEBYKAN_FORWARD_CASE)
#undef CHEBYKAN_FORWARD_CASE
    }
    return false;
}

bool fast_backward_table(const float* x, const float* C, const float* dy, const float* lut, int n, float* dx,
                         float* dC, int64_t B, int I, int O, int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d) || !table_fits(d, n)) return false;
    if (backward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    const TableBasis::Args ba{lut, n};
    switch (d) {
#define CHEBYKAN_BACKWARD_CASE(k) \
    case k: degree_backward<k, TableBasis>(x, C, dy, dx, dC, (int)B, I, O, ws, ba, s); return true;
        CHEBYKAN_FOR_EACH_TABLE_DEGREE(CHEBYKAN_BACKWARD_CASE)
#undef CHEBYKAN_BACKWARD_CASE
    }
    return false;
}

bool fast_backward_table2(const float* x, const float* C, const float* dy, const float* lut, const float* dlut, int n,
                          float* dx, float* dC, int64_t B, int I, int O, int d, void* ws, hipStream_t s)
{
    // both tables ride along in LDS: twice the bytes of the plain table variant
    if (!shape_fits(B, I, O, d) || !table_degree_specialised(d) || n < 2 ||
        2 * (int64_t)n * (d + 1) * (int64_t)sizeof(float) > TABLE_LDS_BYTES)
        return false;
    if (backward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    const DerivTableBasis::Args ba{lut, dlut, n};
    switch (d) {
#define CHEBYKAN_BACKWARD_CASE(k) \
    case k: degree_backward<k, DerivTableBasis>(x, C, dy, dx, dC, (int)B, I, O, ws, ba, s); return true;
        CHEBYKAN_FOR_EACH_TABLE_DEGREE(CHEBYKAN_BACKWARD_CASE)
#undef CHEBYKAN_BACKWARD_CASE
    }
    return false;
}

// ---- forward of a narrow stack in one launch
// Eligible: at least two layers, every width after the input at most 64 (a 128-row tile of one
// layer's output is the next layer's whole input tile), enough rows to fill the GPU with one
// workgroup per 128 rows, vector loads possible for every matrix-core layer; a last layer of
// 1..4 outputs is finished on the vector ALUs.
bool chain_eligible(int n_layers, const int* widths, int d, int64_t B, const float* const* C)
{
    if (!chain_degree(d) || n_layers < 2 || n_layers > CHAIN_MAX_LAYERS) return false;
    if ((B < 128 * 256 && !(test_hooks() & TEST_CHAIN_ANY_BATCH)) || B > 0x7fffffff) return false;
    if ((int64_t)B * (widths[0] > CHAIN_WIDTH ? widths[0] : CHAIN_WIDTH) >= ((int64_t)1 << 30)) return false;
    for (int l = 0; l < n_layers; ++l) {
        const int O = widths[l + 1];
        if (O > CHAIN_WIDTH || widths[l] > 65535) return false;
        const bool narrow_last = l == n_layers - 1 && O <= 4;
        if (!narrow_last && (!aligned16(C[l]) || ((int64_t)O * (d + 1)) % 4 != 0)) return false;
    }
    return true;
}

bool fast_chain_forward(int n_layers, const int* widths, int d, int64_t B, const float* const* C, float* const* act,
                        hipStream_t s)
{
    if (!chain_eligible(n_layers, widths, d, B, C)) return false;
    ChainArgs a;
    a.n_layers = n_layers;
    for (int l = 0; l < n_layers; ++l) a.C[l] = C[l];
    for (int l = 0; l <= n_layers; ++l) { a.act[l] = act[l]; a.width[l] = widths[l]; }
    switch (d) {
#define CHEBYKAN_CHAIN_CASE(k) case k: degree_chain_forward<k>(a, (int)B, s); return true;
        CHEBYKAN_FOR_EACH_CHAIN_DEGREE(CHEBYKAN_CHAIN_CASE)
#undef CHEBYKAN_CHAIN_CASE
    }
    return false;
}

// ---- backward of a stack: the layers' kernels one after the other, every slice sum in one launch at the end.
// Each layer gets its own 256-byte aligned region of the workspace, because its partials now live until that
// last launch.  False (nothing enqueued) when a layer has no specialised kernels.
static size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

size_t stack_backward_workspace_bytes(int n_layers, const int* widths, int d, int64_t B)
{
    size_t total = 0;
    for (int l = 0; l < n_layers; ++l) total += align256(backward_workspace_bytes(B, widths[l], widths[l + 1], d));
    return total;
}

bool fast_stack_backward(int n_layers, const int* widths, int d, int64_t B, const float* const* C,
                         const float* const* act, float* const* grad, float* const* dC, void* ws, hipStream_t s)
{
    if (n_layers > COMBINE_MAX_JOBS || !degree_specialised(d) || B <= 0) return false;
    for (int l = 0; l < n_layers; ++l)
        if (!shape_fits(B, widths[l], widths[l + 1], d)) return false;
    CombineArgs jobs;
    jobs.n_jobs = 0;
    char* region = static_cast<char*>(ws);
    for (int l = n_layers - 1; l >= 0; --l) {
        // dC of this layer and the whole backward of a few-inputs layer below it: one launch for both
        if (l >= 1 && dC[l] && dC[l - 1] && grad[l - 1] && jobs.n_jobs + 2 <= COMBINE_MAX_JOBS &&
            pair_eligible(B, widths[l], widths[l + 1], widths[l - 1], d)) {
            const ScopedLayer layer(l);
            if (!fast_backward(act[l], C[l], grad[l + 1], grad[l], nullptr, B, widths[l], widths[l + 1], d, region, s))
                return false;   // cannot happen after the checks above
            PairArgs a;
            a.x_up = act[l]; a.dy_up = grad[l + 1]; a.dC_up = dC[l]; a.ws_up = reinterpret_cast<float*>(region);
            a.I_up = widths[l]; a.O_up = widths[l + 1]; a.layer_up = l;
            region += align256(backward_workspace_bytes(B, widths[l], widths[l + 1], d));
            a.x_lo = act[l - 1]; a.C_lo = C[l - 1]; a.dy_lo = grad[l]; a.dx_lo = grad[l - 1]; a.dC_lo = dC[l - 1];
            a.ws_lo = reinterpret_cast<float*>(region);
            a.I_lo = widths[l - 1]; a.O_lo = widths[l]; a.B = (int)B;
            region += align256(backward_workspace_bytes(B, widths[l - 1], widths[l], d));
            switch (d) {
#define CHEBYKAN_PAIR_CASE(k) case k: degree_pair_backward<k>(a, &jobs.job[jobs.n_jobs], s); break;
                CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_PAIR_CASE)
#undef CHEBYKAN_PAIR_CASE
            }
            jobs.n_jobs += 2;
            --l;                // the lower layer is done as well
            continue;
        }
        CombineJob job{nullptr, nullptr, 0, 0, 0, 0, 0, 0};
        g_deferred_combine = &job;
        const ScopedLayer layer(l);
        const bool ok = fast_backward(act[l], C[l], grad[l + 1], grad[l], dC[l], B, widths[l], widths[l + 1], d, region, s);
        g_deferred_combine = nullptr;
        if (!ok) return false;   // cannot happen after the checks above; nothing more is enqueued
        if (job.partial) jobs.job[jobs.n_jobs++] = job;
        region += align256(backward_workspace_bytes(B, widths[l], widths[l + 1], d));
    }
    switch (d) {
#define CHEBYKAN_COMBINE_CASE(k) case k: degree_stack_combine<k>(jobs, s); break;
        CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_COMBINE_CASE)
#undef CHEBYKAN_COMBINE_CASE
    }
    return true;
}

// ---- other bases: same plans and workspace, another basis policy
template <class Basis>
static bool family_forward(const float* x, const float* C, float* y, int64_t B, int I, int O, int d, void* ws,
                           hipStream_t s)
{
    const typename Basis::Args ba{};
    switch (d) {
#define CHEBYKAN_CASE(k) case k: degree_forward<k, Basis>(x, C, y, (int)B, I, O, ws, ba, s); return true;
        CHEBYKAN_FOR_EACH_FOURIER_DEGREE(CHEBYKAN_CASE)
#undef CHEBYKAN_CASE
    }
    if constexpr (!std::is_same<Basis, FourierBasis>::value) {
        switch (d) {
            case 3: degree_forward<3, Basis>(x, C, y, (int)B, I, O, ws, ba, s); return true;
            case 5: degree_forward<5, Basis>(x, C, y, (int)B, I, O, ws, ba, s); return true;
        }
    }
    return false;
}

template <class Basis>
static bool family_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int64_t B,
                            int I, int O, int d, void* ws, hipStream_t s)
{
    const typename Basis::Args ba{};
    switch (d) {
#define CHEBYKAN_CASE(k) case k: degree_backward<k, Basis>(x, C, dy, dx, dC, (int)B, I, O, ws, ba, s); return true;
        CHEBYKAN_FOR_EACH_FOURIER_DEGREE(CHEBYKAN_CASE)
#undef CHEBYKAN_CASE
    }
    if constexpr (!std::is_same<Basis, FourierBasis>::value) {
        switch (d) {
            case 3: degree_backward<3, Basis>(x, C, dy, dx, dC, (int)B, I, O, ws, ba, s); return true;
            case 5: degree_backward<5, Basis>(x, C, dy, dx, dC, (int)B, I, O, ws, ba, s); return true;
        }
    }
    return false;
}

bool fast_forward_family(int kind, const float* x, const float* C, float* y, int64_t B, int I, int O, int d,
                         void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d)) return false;
    if (forward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    switch (kind) {
        case 1: return family_forward<LegendreBasis>(x, C, y, B, I, O, d, ws, s);
        case 2: return family_forward<HermiteBasis>(x, C, y, B, I, O, d, ws, s);
        case 3: return family_forward<FourierBasis>(x, C, y, B, I, O, d, ws, s);
    }
    return false;
}

bool fast_backward_family(int kind, const float* x, const float* C, const float* dy, float* dx, float* dC,
                          int64_t B, int I, int O, int d, void* ws, hipStream_t s)
{
    if (!shape_fits(B, I, O, d)) return false;
    if (backward_workspace_bytes(B, I, O, d) > 0 && !ws) return false;
    switch (kind) {
        case 1: return family_backward<LegendreBasis>(x, C, dy, dx, dC, B, I, O, d, ws, s);
        case 2: return family_backward<HermiteBasis>(x, C, dy, dx, dC, B, I, O, d, ws, s);
        case 3: return family_backward<FourierBasis>(x, C, dy, dx, dC, B, I, O, d, ws, s);
    }
    return false;
}

}  // namespace chebykan
