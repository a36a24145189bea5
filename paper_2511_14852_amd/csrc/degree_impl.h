// Launch code of the specialised kernels for ONE degree.  Included by the per-degree
// translation units (deg_NN.hip), each of which instantiates degree_forward<D> and
// degree_backward<D> for its degree; the dispatcher only sees their declarations.
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>

#include "chain_kernels.h"
#include "launch.h"
#include "mfma_kernels.h"
#include "narrow_in_kernels.h"
#include "narrow_kernels.h"
#include "plans.h"

namespace chebykan {

// A workgroup may use the whole 160 KiB of a compute unit when a basis table rides along.
constexpr int MAX_LDS_BYTES = 160 * 1024;

// LDS bytes the basis policy adds to a kernel's own tiles (the staged table; 0 for the recurrences).
template <class Basis>
inline size_t basis_lds_bytes(const typename Basis::Args& ba, int K)
{
    if constexpr (Basis::kTable) return (size_t)Basis::kTableRows * ba.n * K * sizeof(float);
    else { (void)ba; (void)K; return 0; }
}

// When a stack's backward pass is running, the per-layer launch code records each layer's slice sum
// here instead of launching it; the stack code then runs all of them in one launch.  Null otherwise.
extern thread_local CombineJob* g_deferred_combine;

// Many slices of a small tensor (coefficient gradients of narrow layers): 32 slice groups.
// Few slices of a large tensor (split forward): 4 groups, 64 consecutive elements per block.
// `run` / `stride`: the output as a window of a larger tensor (see sum_slices_kernel); run = 0 means out[e].
inline void launch_sum_slices(const float* partial, float* out, int64_t n, int slices, hipStream_t s, int64_t run = 0,
                              int64_t stride = 0)
{
    if (run <= 0) { run = n; stride = 0; }
    // few large planes: plain streaming with 16-byte accesses; small sums are latency-bound and keep the
    // many-block form (c4's 16000 x 257 x 2 planes 22 -> 12 us; 16K elements x 4 planes measured 0.4 us slower)
    if (slices <= 8 && n >= ((int64_t)1 << 20) && run == n) {
        const dim3 grid((unsigned)((n + 1023) / 1024));
        if (n % 4 == 0 && aligned16(partial) && aligned16(out))
            launch<sum_few_slices_kernel<4>, 0, Tags<Int<4>>>(grid, dim3(256), 0, s, partial, out, n, slices);
        else
            launch<sum_few_slices_kernel<1>, 0, Tags<Int<1>>>(grid, dim3(256), 0, s, partial, out, n, slices);
    } else if (slices > 16)
        launch<sum_slices_kernel<32>, 0, Tags<Int<32>>>(dim3((unsigned)((n + 7) / 8)), dim3(256), 32 * 9 * sizeof(float), s, partial, out, n,
                                      slices, run, stride);
    else
        launch<sum_slices_kernel<4>, 0, Tags<Int<4>>>(dim3((unsigned)((n + 63) / 64)), dim3(256), 4 * 65 * sizeof(float), s, partial, out, n,
                                     slices, run, stride);
}

// ------------------------------------------------------------ narrow layers
template <int D, int O, class Basis>
void launch_narrow_fwd(const float* x, const float* C, float* y, int B, int I, const typename Basis::Args& ba, hipStream_t s,
                       int o_stride, int o_begin)
{
    const NarrowPlan p = plan_narrow(B, I, NARROW_FWD_WGS);
    launch<narrow_fwd_kernel<D, O, Basis>, MAX_LDS_BYTES, Tags<Int<D>, Int<O>, Basis>>(
        dim3((unsigned)p.slices), dim3(NARROW_THREADS),
        narrow_fwd_lds_floats(I, O, D + 1) * sizeof(float) + basis_lds_bytes<Basis>(ba, D + 1), s, x, C, y, B, I, p.G,
        p.rows_per_wg, ba, o_stride, o_begin);
}

template <int D, int O, class Basis>
void launch_narrow_bwd(const float* x, const float* C, const float* dy, float* dx, float* dC, float* partial,
                       int B, int I, const typename Basis::Args& ba, hipStream_t s, int o_stride, int o_begin)
{
    const NarrowPlan p = plan_narrow(B, I, NARROW_BWD_WGS);
    const int blocks_i = (I + p.G - 1) / p.G;
    launch<narrow_bwd_kernel<D, O, Basis>, MAX_LDS_BYTES, Tags<Int<D>, Int<O>, Basis>>(
        dim3((unsigned)p.slices, (unsigned)blocks_i), dim3(NARROW_THREADS),
        narrow_bwd_lds_floats(O, D + 1) * sizeof(float) + basis_lds_bytes<Basis>(ba, D + 1), s, x, C, dy, dx,
        dC ? partial : nullptr, B, I, p.G, p.rows_per_wg, ba, o_stride, o_begin);
    if (dC) {
        if (g_deferred_combine && o_stride == O)
            *g_deferred_combine = CombineJob{partial, dC, I, O, p.slices, 1, (int64_t)I * O * (D + 1), 0};
        else {
            // the partials are compact [slice][i][o][k]; in a window, dC's runs of O*K values lie o_stride*K apart
            const ScopedOps ops(OP_DC | OP_SUM);
            launch_sum_slices(partial, dC + (int64_t)o_begin * (D + 1), (int64_t)I * O * (D + 1), p.slices, s,
                              (int64_t)O * (D + 1), (int64_t)o_stride * (D + 1));
        }
    }
}

// O columns starting at o_begin of a layer with o_stride outputs (a narrow layer: o_stride = O, o_begin = 0)
template <int D, class Basis>
void narrow_fwd_by_out(const float* x, const float* C, float* y, int B, int I, int O, const typename Basis::Args& ba, hipStream_t s,
                       int o_stride, int o_begin)
{
    switch (O) {
        case 1: launch_narrow_fwd<D, 1, Basis>(x, C, y, B, I, ba, s, o_stride, o_begin); break;
        case 2: launch_narrow_fwd<D, 2, Basis>(x, C, y, B, I, ba, s, o_stride, o_begin); break;
        case 3: launch_narrow_fwd<D, 3, Basis>(x, C, y, B, I, ba, s, o_stride, o_begin); break;
        default: launch_narrow_fwd<D, 4, Basis>(x, C, y, B, I, ba, s, o_stride, o_begin); break;
    }
}

template <int D, class Basis>
void narrow_bwd_by_out(const float* x, const float* C, const float* dy, float* dx, float* dC, float* partial, int B,
                       int I, int O, const typename Basis::Args& ba, hipStream_t s, int o_stride, int o_begin)
{
    switch (O) {
        case 1: launch_narrow_bwd<D, 1, Basis>(x, C, dy, dx, dC, partial, B, I, ba, s, o_stride, o_begin); break;
        case 2: launch_narrow_bwd<D, 2, Basis>(x, C, dy, dx, dC, partial, B, I, ba, s, o_stride, o_begin); break;
        case 3: launch_narrow_bwd<D, 3, Basis>(x, C, dy, dx, dC, partial, B, I, ba, s, o_stride, o_begin); break;
        default: launch_narrow_bwd<D, 4, Basis>(x, C, dy, dx, dC, partial, B, I, ba, s, o_stride, o_begin); break;
    }
}

// ------------------------------------------------------------------ forward
template <int D, int BN, int VEC, class Basis, int RB = 4>
void launch_fwd(const float* x, const float* C, float* out, int B, int I, int O, int tiles_o, int o_begin,
                const FwdPlan& p, const typename Basis::Args& ba, hipStream_t s)
{
    using Cfg = FwdCfg<D, BN, forward_chunk_features(D), VEC, RB>;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * tiles_o;
    launch<fwd_mfma_kernel<Cfg, Basis>, Basis::kTable ? MAX_LDS_BYTES : Cfg::LDS_BYTES, Tags<Cfg, Basis>>(
        dim3((unsigned)tiles, (unsigned)p.splits), dim3(MFMA_THREADS), Cfg::LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1), s,
        x, C, out, B, I, O, tiles_o, o_begin, p.chunks_per_split, ba);
}

template <int D, class Basis>
void pick_fwd(const float* x, const float* C, float* y, float* partial, int B, int I, int O, const typename Basis::Args& ba, hipStream_t s)
{
    // coefficient slabs are copied with 16-byte loads: global memory only needs 4-byte aligned addresses for
    // them, and the LDS side of the copy stays 16-byte aligned
    const FwdPlan p = plan_forward(B, I, O, D);
    float* out = p.splits > 1 ? partial : y;
    if (O <= 64) {
        launch_fwd<D, 64, 4, Basis>(x, C, out, B, I, O, 1, 0, p, ba, s);
    } else {
        const OutTiling t = out_tiling(I, O, D);
        // batches of at most 64 rows (the paper's operator shapes): waves side by side, no MFMAs on
        // row blocks that are all padding; built for the exact basis at the degrees those shapes use
        constexpr bool small_batch_built = D >= 7 && std::is_same<Basis, ExactBasis>::value;
        bool done = false;
        if constexpr (small_batch_built) {
            if (B <= 32) { launch_fwd<D, 128, 4, Basis, 1>(x, C, out, B, I, O, t.wide_tiles, 0, p, ba, s); done = true; }
            else if (B <= 64) { launch_fwd<D, 128, 4, Basis, 2>(x, C, out, B, I, O, t.wide_tiles, 0, p, ba, s); done = true; }
        }
        const float wide_share = t.tail_begin >= 0 ? (float)t.tail_begin / (float)O : 1.0f;
        if (!done) {
            const ScopedShare share(wide_share);
            launch_fwd<D, 128, 4, Basis>(x, C, out, B, I, O, t.wide_tiles, 0, p, ba, s);
        }
        if (t.tail_kind == 1) {
            const ScopedShare share(1.0f - wide_share);
            launch_fwd<D, 64, 4, Basis>(x, C, out, B, I, O, 1, t.tail_begin, p, ba, s);
        }
    }
    if (p.splits > 1) {
        const ScopedOps ops(OP_FWD | OP_SUM);
        launch_sum_slices(partial, y, (int64_t)B * O, p.splits, s);
    }
    if (O > 64) {
        // 1..4 columns beyond the 128-wide tiles: streamed, straight into y (after the plane sum, which
        // passes over those columns with whatever the planes held there)
        const OutTiling t = out_tiling(I, O, D);
        if (t.tail_kind == 2) {
            const ScopedShare share(1.0f - (float)t.tail_begin / (float)O);
            narrow_fwd_by_out<D, Basis>(x, C, y, B, I, O - t.tail_begin, ba, s, O, t.tail_begin);
        }
    }
}

// --------------------------------------------------------------------- dC
template <int D>
void launch_dC_combine(const float* partial, float* dC, int I, int O, int slices, hipStream_t s, int o_count = -1)
{
    const ScopedOps ops(OP_DC | OP_SUM);
    if (o_count < 0) o_count = O;      // columns the partials hold (fewer when a streamed tail makes the rest)
    // small sums are latency-bound and gain from sharing one launch; large ones run at once
    if (g_deferred_combine && o_count == O && (int64_t)((O + 31) / 32) * I <= 512) {
        *g_deferred_combine = CombineJob{partial, dC, I, O, slices, 0, 0, 0};
        return;
    }
    const dim3 grid((unsigned)((o_count + 31) / 32), (unsigned)I);
    constexpr int lds32 = 1024 * ((D + 1) | 1) * (int)sizeof(float), lds8 = 256 * ((D + 1) | 1) * (int)sizeof(float);
    if (slices > 32)
        launch<dC_combine_kernel<D, 32>, lds32, Tags<Int<D>, Int<32>>>(grid, dim3(1024), lds32, s, partial, dC, I, O, o_count, slices);
    else
        launch<dC_combine_kernel<D, 8>, lds8, Tags<Int<D>, Int<8>>>(grid, dim3(256), lds8, s, partial, dC, I, O, o_count, slices);
}

template <int D, int BN, int VEC, int BIC, class Basis>
void launch_dC(const float* x, const float* dy, float* partial, float* direct, int B, int I, int O, int tiles_o,
               int o_begin, const DcPlan& p, const typename Basis::Args& ba, hipStream_t s)
{
    using Cfg = DcCfg<D, BN, VEC, BIC>;
    constexpr int kAllow = Basis::kTable ? MAX_LDS_BYTES
                                         : (Cfg::DIRECT_LDS_BYTES > Cfg::LDS_BYTES ? Cfg::DIRECT_LDS_BYTES : Cfg::LDS_BYTES);
    const int tiles_i = (I + Cfg::BIC - 1) / Cfg::BIC;
    size_t lds_bytes = Cfg::LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1);
    if (direct && lds_bytes < (size_t)Cfg::DIRECT_LDS_BYTES) lds_bytes = Cfg::DIRECT_LDS_BYTES;   // the epilogue's layout turn
    launch<dC_mfma_kernel<Cfg, Basis>, kAllow, Tags<Cfg, Basis>>(dim3((unsigned)((int64_t)tiles_i * tiles_o * p.slices)), dim3(MFMA_THREADS),
                                               lds_bytes, s, x, dy, partial, B, I, O, tiles_o, o_begin, tiles_i, p.slices,
                                               p.rows_per_slice, ba, direct);
}

template <int D, int BIC, class Basis>
void pick_dC_tile(const float* x, const float* dy, float* partial, float* direct, int B, int I, int O, const DcPlan& p,
                  const typename Basis::Args& ba, hipStream_t s)
{
    // dy rows are copied with 16-byte loads at any 4-byte aligned address (see pick_fwd)
    if (p.bn == 64) {
        launch_dC<D, 64, 4, BIC, Basis>(x, dy, partial, direct, B, I, O, 1, 0, p, ba, s);
    } else {
        const OutTiling t = out_tiling(I, O, D);
        const float wide_share = t.tail_begin >= 0 ? (float)t.tail_begin / (float)O : 1.0f;
        {
            const ScopedShare share(wide_share);
            launch_dC<D, 128, 4, BIC, Basis>(x, dy, partial, direct, B, I, O, t.wide_tiles, 0, p, ba, s);
        }
        if (t.tail_kind == 1) {
            const ScopedShare share(1.0f - wide_share);
            launch_dC<D, 64, 4, BIC, Basis>(x, dy, partial, direct, B, I, O, 1, t.tail_begin, p, ba, s);
        }
    }
}

template <int D, class Basis>
void pick_dC(const float* x, const float* dy, float* dC, float* partial, int B, int I, int O, const DcPlan& p,
             const typename Basis::Args& ba, hipStream_t s)
{
    // With one batch slice the tiles are final: the slice kernel writes dC itself, in the caller's
    // layout, and the slice sum is not launched.  Only with enough tiles: each workgroup turns its
    // own tile, and a handful of workgroups do that slower than the many blocks of the sum kernel
    // (measured with the element-wise copy: 3 and 6 tiles lose 1-4 us, 128 and 824 tiles gain 4 and 9 us).
    const int bic = dc_tile_features_for(I, D);
    const int64_t tiles = (int64_t)((I + bic - 1) / bic) * ((O + p.bn - 1) / p.bn);
    // With 16-byte aligned runs the tile leaves as whole float4 stores, which wins at any tile count.
    // (The test hook TEST_DIRECT_DC takes this path at any tile count: tests of that epilogue on small inputs.)
    const bool vector_out = O % 4 == 0 && aligned16(dC);
    float* direct = (p.slices == 1 && (tiles >= 64 || vector_out || (test_hooks() & TEST_DIRECT_DC))) ? dC : nullptr;
    if constexpr (D == 6) {
        if (dc_tile_features_for(I, D) == 16) pick_dC_tile<D, 16, Basis>(x, dy, partial, direct, B, I, O, p, ba, s);
        else pick_dC_tile<D, dc_tile_features(D), Basis>(x, dy, partial, direct, B, I, O, p, ba, s);
    } else {
        pick_dC_tile<D, dc_tile_features(D), Basis>(x, dy, partial, direct, B, I, O, p, ba, s);
    }
    const OutTiling t = out_tiling(I, O, D);
    const bool streamed_tail = p.bn == 128 && t.tail_kind == 2;
    if (!direct) launch_dC_combine<D>(partial, dC, I, O, p.slices, s, streamed_tail ? t.tail_begin : O);
    if (streamed_tail) {
        // the 1..4 columns beyond the 128-wide tiles: per-workgroup partials behind those of the tiles, then a sum
        // into the window of dC
        const ScopedShare share(1.0f - (float)t.tail_begin / (float)O);
        float* tail_partial = partial + (size_t)p.slices * I * (D + 1) * O;
        narrow_bwd_by_out<D, Basis>(x, nullptr, dy, nullptr, dC, tail_partial, B, I, O - t.tail_begin, ba, s, O, t.tail_begin);
    }
}

// --------------------------------------------------------------------- dx
template <int D, int NB, int VEC, class Basis, int RB = 4>
void launch_dx(const float* x, const float* C, const float* dy, float* dx, float* partial, int B, int I, int O,
               const DxPlan& p, const typename Basis::Args& ba, hipStream_t s)
{
    using Cfg = DxCfg<D, NB, VEC, RB>;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * p.feature_tiles;
    launch<dx_mfma_kernel<Cfg, Basis>, Basis::kTable ? MAX_LDS_BYTES : Cfg::LDS_BYTES, Tags<Cfg, Basis>>(
        dim3((unsigned)tiles, (unsigned)p.split.splits), dim3(MFMA_THREADS), Cfg::LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1),
        s, x, C, dy, p.split.splits > 1 ? partial : dx, B, I, O, p.feature_tiles, p.split.chunks_per_split, 0, ba);
}

// The few features from p.tail_begin on, beside a feature-per-lane launch over the full tiles (see DxPlan).
template <int D, int NB, class Basis>
void launch_dx_tail(const float* x, const float* C, const float* dy, float* dx, int B, int I, int O,
                    const DxPlan& p, const typename Basis::Args& ba, hipStream_t s)
{
    using Cfg = DxCfg<D, NB, 4, 4>;
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * p.tail_tiles;
    launch<dx_mfma_kernel<Cfg, Basis>, Basis::kTable ? MAX_LDS_BYTES : Cfg::LDS_BYTES, Tags<Cfg, Basis>>(
        dim3((unsigned)tiles, 1u), dim3(MFMA_THREADS), Cfg::LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1),
        s, x, C, dy, dx, B, I, O, p.tail_tiles, (O + Cfg::BO - 1) / Cfg::BO, p.tail_begin, ba);
}

template <int D, int VEC, class Basis>
void launch_dx2(const float* x, const float* C, const float* dy, float* dx, float* partial, int B, int I, int O,
                const DxPlan& p, const typename Basis::Args& ba, hipStream_t s)
{
    using Cfg = Dx2Cfg<D, VEC>;
    static_assert(Cfg::BO == (D <= 4 ? 32 : 16), "plan_dx assumes this chunk width");
    const int64_t tiles = (int64_t)((B + Cfg::BM - 1) / Cfg::BM) * p.feature_tiles;
    launch<dx2_mfma_kernel<Cfg, Basis>, Basis::kTable ? MAX_LDS_BYTES : Cfg::LDS_BYTES, Tags<Cfg, Basis>>(
        dim3((unsigned)tiles, (unsigned)p.split.splits), dim3(MFMA_THREADS), Cfg::LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1),
        s, x, C, dy, p.split.splits > 1 ? partial : dx, B, I, O, p.feature_tiles, p.split.chunks_per_split, p.tail_begin, ba);
}

template <int D, class Basis>
void pick_dx(const float* x, const float* C, const float* dy, float* dx, float* partial, int B, int I, int O,
             const typename Basis::Args& ba, hipStream_t s)
{
    // dy rows and coefficient runs are copied with 16-byte loads at any 4-byte aligned address (see pick_fwd)
    const DxPlan p = plan_dx(B, I, O, D);
    bool done = false;
    if constexpr (D <= 6) {   // the feature-per-lane kernel exists for these degrees only
        if (p.per_lane) {
            if (p.tail_begin < I) {
                // full tiles here, the remaining features from a packed-column launch; the work share of
                // each goes into the timing report
                {
                    ScopedShare share((float)p.tail_begin / (float)I);
                    launch_dx2<D, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s);
                }
                ScopedShare share((float)(I - p.tail_begin) / (float)I);
                if (p.tail_nb == 1) launch_dx_tail<D, 1, Basis>(x, C, dy, dx, B, I, O, p, ba, s);
                else launch_dx_tail<D, 2, Basis>(x, C, dy, dx, B, I, O, p, ba, s);
            } else {
                launch_dx2<D, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s);
            }
            done = true;
        }
    }
    // batches of at most 64 rows: one column block per wave (see DxCfg); built like the forward variant
    if constexpr (D >= 7 && std::is_same<Basis, ExactBasis>::value) {
        if (!done && B <= 64) {
            const bool one = B <= 32;
            switch (p.nb) {
                case 1: one ? launch_dx<D, 1, 4, Basis, 1>(x, C, dy, dx, partial, B, I, O, p, ba, s)
                            : launch_dx<D, 1, 4, Basis, 2>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
                case 2: one ? launch_dx<D, 2, 4, Basis, 1>(x, C, dy, dx, partial, B, I, O, p, ba, s)
                            : launch_dx<D, 2, 4, Basis, 2>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
                case 3: one ? launch_dx<D, 3, 4, Basis, 1>(x, C, dy, dx, partial, B, I, O, p, ba, s)
                            : launch_dx<D, 3, 4, Basis, 2>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
                default: one ? launch_dx<D, 4, 4, Basis, 1>(x, C, dy, dx, partial, B, I, O, p, ba, s)
                             : launch_dx<D, 4, 4, Basis, 2>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
            }
            done = true;
        }
    }
    if (!done) {
        switch (p.nb) {
            case 1: launch_dx<D, 1, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
            case 2: launch_dx<D, 2, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
            case 3: launch_dx<D, 3, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
            default: launch_dx<D, 4, 4, Basis>(x, C, dy, dx, partial, B, I, O, p, ba, s); break;
        }
    }
    if (p.split.splits > 1) {
        const ScopedOps ops(OP_DX | OP_SUM);
        launch_sum_slices(partial, dx, (int64_t)B * I, p.split.splits, s);
    }
}

// ------------------------------------------------------------ two operations in one launch
// Stack backward: the coefficient gradient of layer `up` (out <= 64, several batch slices) together with the
// whole backward pass of the few-inputs layer below it (see dC_with_few_inputs_kernel).  The caller has
// checked pair_eligible() and has already launched dx of the upper layer.  Both slice sums are recorded in
// `jobs` (two entries) for the stack's single combine launch.
template <int D, int BIC>
void launch_pair(const PairArgs& a, const DcPlan& p, const NarrowInPlan& q, hipStream_t s)
{
    using Cfg = DcCfg<D, 64, 4, BIC>;
    constexpr int lds = Cfg::LDS_BYTES > NIN_LDS_BYTES ? Cfg::LDS_BYTES : NIN_LDS_BYTES;
    const int tiles_i = (a.I_up + BIC - 1) / BIC;
    const DcSliceArgs up{a.x_up, a.dy_up, a.ws_up, a.B, a.I_up, a.O_up, 1, 0, tiles_i, p.slices, p.rows_per_slice};
    const FewInputsArgs lo{a.x_lo, a.C_lo, a.dy_lo, a.dx_lo, a.ws_lo, a.B, a.I_lo, a.O_lo, q.rows_per_slice};
    const ScopedLayer layer(a.layer_up);
    const ScopedOps ops(OP_DC);
    const ScopedSecond second(a.layer_up - 1, OP_DX | OP_DC);
    launch<dC_with_few_inputs_kernel<Cfg, D>, lds, Tags<Cfg, Int<D>>>(dim3((unsigned)(q.slices + tiles_i * p.slices)), dim3(MFMA_THREADS),
                                                                      (size_t)lds, s, up, lo, q.slices);
}

template <int D>
void degree_pair_backward(const PairArgs& a, CombineJob* jobs, hipStream_t s)
{
    const DcPlan p = plan_dC(a.B, a.I_up, a.O_up, D);
    const NarrowInPlan q = plan_narrow_in(a.B);
    if constexpr (D == 6) {
        if (dc_tile_features_for(a.I_up, D) == 16) launch_pair<D, 16>(a, p, q, s);
        else launch_pair<D, dc_tile_features(D)>(a, p, q, s);
    } else {
        launch_pair<D, dc_tile_features(D)>(a, p, q, s);
    }
    jobs[0] = CombineJob{a.ws_up, a.dC_up, a.I_up, a.O_up, p.slices, 0, 0, 0};
    jobs[1] = CombineJob{a.ws_lo, a.dC_lo, a.I_lo, a.O_lo, q.slices, 0, 0, 0};
}

// All deferred slice sums of a stack in one launch.
template <int D>
void degree_stack_combine(CombineArgs& a, hipStream_t s)
{
    const ScopedLayer all_layers(-1);
    const ScopedOps ops(OP_DC | OP_SUM);
    int blocks = 0;
    for (int q = 0; q < a.n_jobs; ++q) {
        a.job[q].first_block = blocks;
        blocks += combine_job_blocks(a.job[q]);
    }
    if (blocks == 0) return;
    constexpr int lds_bytes = 1024 * ((D + 1) | 1) * (int)sizeof(float);
    launch<stack_combine_kernel<D>, lds_bytes, Tags<Int<D>>>(dim3((unsigned)blocks), dim3(1024), lds_bytes, s, a);
}

// ------------------------------------------------------------ fused narrow stack
// Forward of a whole stack in one launch; the caller has checked chain_eligible().
template <int D>
void degree_chain_forward(const ChainArgs& a, int B, hipStream_t s)
{
    const ScopedLayer all_layers(-1);
    const ScopedOps ops(OP_FWD);
    launch<fwd_chain_kernel<D>, chain_lds_bytes<D>(), Tags<Int<D>>>(dim3((unsigned)((B + 127) / 128)), dim3(MFMA_THREADS),
                                                      (size_t)chain_lds_bytes<D>(), s, a, B);
}

// ------------------------------------------------------- per-degree entry points
// `ws` is the caller's workspace (partial outputs of a split forward contraction; partial
// coefficient gradients of the batch slices).
template <int D, class Basis>
void degree_forward(const float* x, const float* C, float* y, int B, int I, int O, void* ws, const typename Basis::Args& ba, hipStream_t s)
{
    const ScopedOps ops(OP_FWD);
    if (use_narrow(B, I, O, D)) narrow_fwd_by_out<D, Basis>(x, C, y, B, I, O, ba, s, O, 0);
    else pick_fwd<D, Basis>(x, C, y, static_cast<float*>(ws), B, I, O, ba, s);
}

template <int D, class Basis>
void degree_backward(const float* x, const float* C, const float* dy, float* dx, float* dC, int B, int I, int O,
                     void* ws, const typename Basis::Args& ba, hipStream_t s)
{
    float* partial = static_cast<float*>(ws);
    const ScopedOps both((dx ? OP_DX : 0) | (dC ? OP_DC : 0));
    if (use_narrow(B, I, O, D)) {
        narrow_bwd_by_out<D, Basis>(x, C, dy, dx, dC, partial, B, I, O, ba, s, O, 0);
        return;
    }
    if (dx && dC && use_narrow_in(B, I, O, D)) {   // few inputs, both gradients wanted: one kernel for both
        const NarrowInPlan p = plan_narrow_in(B);
        launch<bwd_narrow_in_kernel<D, Basis>, Basis::kTable ? MAX_LDS_BYTES : NIN_LDS_BYTES, Tags<Int<D>, Basis>>(
            dim3((unsigned)p.slices), dim3(MFMA_THREADS), NIN_LDS_BYTES + basis_lds_bytes<Basis>(ba, D + 1), s, x, C, dy, dx,
            dC ? partial : nullptr, B, I, O, p.rows_per_slice, ba);
        if (dC) launch_dC_combine<D>(partial, dC, I, O, p.slices, s);
        return;
    }
    // the dx partials are summed before the dC kernel reuses the workspace (same stream)
    if (dx) {
        const ScopedOps ops(OP_DX);
        pick_dx<D, Basis>(x, C, dy, dx, partial, B, I, O, ba, s);
    }
    if (dC) {
        const ScopedOps ops(OP_DC);
        if constexpr (std::is_same<Basis, DerivTableBasis>::value) {
            // the coefficient gradient needs no derivative: the kernels of the plain table variant serve it
            pick_dC<D, TableBasis>(x, dy, dC, partial, B, I, O, plan_dC(B, I, O, D), TableBasis::Args{ba.lut, ba.n}, s);
        } else {
            pick_dC<D, Basis>(x, dy, dC, partial, B, I, O, plan_dC(B, I, O, D), ba, s);
        }
    }
}

}  // namespace chebykan
