// Host-side planning shared by the dispatcher and the per-degree launch code:
// which degrees have specialised kernels, which shapes they take, batch-slice and
// feature-split plans.  No kernels here.
#pragma once
#include <stdint.h>
#include <stdlib.h>

namespace chebykan {

// Degrees with specialised kernels.  Each one is compiled in its own translation unit
// (deg_NN.hip); everything else runs on the any-degree kernels.
#define CHEBYKAN_FOR_EACH_DEGREE(X) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(15) X(24)

inline bool degree_specialised(int d)
{
#define CHEBYKAN_DEGREE_CASE(n) if (d == n) return true;
    CHEBYKAN_FOR_EACH_DEGREE(CHEBYKAN_DEGREE_CASE)
#undef CHEBYKAN_DEGREE_CASE
    return false;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Degrees whose kernels are also built in the table-interpolated form, and the LDS bytes a
// staged table may take next to the largest kernel's own tiles (about 76 KiB of 160).
#define CHEBYKAN_FOR_EACH_TABLE_DEGREE(X) X(2) X(3) X(4) X(5) X(6) X(7) X(8)
constexpr bool table_degree_specialised(int d) { return d >= 2 && d <= 8; }
constexpr int64_t TABLE_LDS_BYTES = 80 * 1024;

// Degrees at which the Legendre / Hermite kernels and (even ones only) the Fourier kernels are built.
#define CHEBYKAN_FOR_EACH_FAMILY_DEGREE(X) X(3) X(4) X(5) X(6) X(8)
#define CHEBYKAN_FOR_EACH_FOURIER_DEGREE(X) X(4) X(6) X(8)
constexpr bool family_degree_specialised(int d) { return d == 3 || d == 4 || d == 5 || d == 6 || d == 8; }
constexpr bool fourier_degree_specialised(int d) { return d == 4 || d == 6 || d == 8; }

// Degrees with a fused narrow-stack forward kernel (its LDS tiles fit twice into a compute unit).
#define CHEBYKAN_FOR_EACH_CHAIN_DEGREE(X) X(3) X(4) X(5) X(6)
constexpr bool chain_degree(int d) { return d >= 3 && d <= 6; }

// Test hooks.  Four plan decisions depend on sizes that only large inputs reach; the host-side
// emulation tests need them on small inputs.  A build with -DCHEBYKAN_TEST_HOOKS reads a bit mask
// from the environment variable CHEBYKAN_TEST_HOOKS once; the product build has no such switch.
constexpr int TEST_CHAIN_ANY_BATCH = 1;   // fuse a narrow stack's forward at any batch size
constexpr int TEST_DIRECT_DC = 2;         // a single-slice dC is written by the slice kernel at any tile count
constexpr int TEST_DC_MIN_256_ROWS = 4;   // small batches keep at least 256 rows per coefficient-gradient slice
constexpr int TEST_DX_TAIL_ANY_SIZE = 8;  // a second input-gradient launch for the last few features at any amount of work
#ifdef CHEBYKAN_TEST_HOOKS
inline int test_hooks()
{
    static const int flags = [] {
        const char* e = getenv("CHEBYKAN_TEST_HOOKS");
        return e ? atoi(e) : 0;
    }();
    return flags;
}
#else
constexpr int test_hooks() { return 0; }
#endif

// Input features per forward chunk: about 28-50 contraction terms per chunk.
constexpr int forward_chunk_features(int d)
{
    return d <= 2 ? 12 : d <= 4 ? 8 : d == 5 ? 6 : d <= 8 ? 4 : 2;
}

inline bool use_narrow_shape(int I, int O, int d) { return O <= 4 && (int64_t)I * O * (d + 1) <= 16384; }

// ------------------------------------------------- layers with very few inputs
// Both gradients of a layer whose (i,k) rows and outputs fit one 64 x 64 tile come from one
// kernel (narrow_in_kernels.h).
inline bool use_narrow_in(int64_t B, int I, int O, int d)
{
    return B >= 1 && I * (d + 1) <= 64 && I <= 16 && O <= 64 && O > 4;
}

struct NarrowInPlan {
    int slices;
    int rows_per_slice;   // multiple of 32
};

inline NarrowInPlan plan_narrow_in(int64_t B)
{
    int64_t rows = (B + 255) / 256;            // one workgroup per compute unit measured best (128..1024 tried)
    if (rows < 128) rows = 128;
    rows = (rows + 31) / 32 * 32;
    NarrowInPlan p;
    p.rows_per_slice = (int)rows;
    p.slices = (int)((B + rows - 1) / rows);
    return p;
}

// Stack backward: the coefficient gradient of a layer with at most 64 outputs and the backward pass of a
// few-inputs layer directly below it can share one launch (both only need dx of the upper layer).  The upper
// layer must go through the matrix-core slice kernel with partials (several slices) and small slice sums.
inline bool pair_eligible(int64_t B, int I_up, int O_up, int I_lo, int d);
struct PairArgs {
    // upper layer: dC only
    const float* x_up;
    const float* dy_up;
    float* dC_up;
    float* ws_up;
    int I_up, O_up, layer_up;
    // lower layer: dx and dC
    const float* x_lo;
    const float* C_lo;
    const float* dy_lo;
    float* dx_lo;
    float* dC_lo;
    float* ws_lo;
    int I_lo, O_lo;
    int B;
};


// Output tiling: 128-wide tiles, except that a remainder beyond a multiple of 128 is handled apart.
// 1..4 left-over columns (257 outputs) go to the streaming kernels of narrow_kernels.h, which cost
// about a tenth of a 64-wide matrix-core tile that would compute 60 unused columns; 5..64 columns
// get one 64-wide tile from a second launch (2 x 128 + 64 computed columns instead of 3 x 128).
constexpr int NARROW_MAX_OUT = 4;
struct OutTiling {
    int wide_tiles;    // 128-wide tiles from column 0
    int tail_begin;    // first column of the tail, or -1
    int tail_kind;     // 0 none, 1 one 64-wide matrix-core tile, 2 streaming kernels
};
inline OutTiling out_tiling(int I, int O, int d)
{
    const int rem = O % 128;
    if (O > 128 && rem >= 1 && rem <= NARROW_MAX_OUT && (int64_t)I * rem * (d + 1) <= 16384)
        return OutTiling{O / 128, (O / 128) * 128, 2};
    if (O > 128 && rem >= 1 && rem <= 64) return OutTiling{O / 128, (O / 128) * 128, 1};
    return OutTiling{(O + 127) / 128, -1, 0};
}

// Time of one launch of `wg` equal workgroups, in units of one workgroup's run time when two share
// a compute unit.  512 are resident at once; one alone on its unit runs in about 0.6 of that time.
inline double launch_rounds(int64_t wg)
{
    if (wg <= 0) return 0.0;
    const int64_t full = wg / 512, rem = wg % 512;
    return (double)full + (rem == 0 ? 0.0 : rem <= 256 ? 0.6 : 1.0);
}

// --------------------------------------------------------------------- dC
struct DcPlan {
    int bn;              // output tile width
    int slices;          // batch slices (partial buffers)
    int rows_per_slice;  // multiple of 32
};

// Batch slices for the coefficient gradient.  512 workgroups are resident at once
// (256 CUs x 2); the slice count is the one with the lowest estimated time (whole rounds
// of resident workgroups times rows per slice, plus the traffic of the partial tensors),
// subject to >= 256 rows per slice and a 512 MiB cap on the partial buffers.
// Input features per coefficient-gradient tile.  128/K features fill the 128 tile rows best,
// but the basis chunk of 32 rows x bic features is generated by 256 threads, and a feature
// count that is a multiple of 8 splits it evenly.  At degree 6 (18 features) the even split (16)
// is taken whenever it does not add a tile.
constexpr int dc_tile_features(int d) { return 128 / (d + 1); }
inline int dc_tile_features_for(int I, int d)
{
    const int full = dc_tile_features(d);
    if (d == 6 && (I + 15) / 16 == (I + full - 1) / full) return 16;
    return full;
}

inline DcPlan plan_dC(int64_t B, int I, int O, int d)
{
    const int K = d + 1;
    DcPlan p;
    p.bn = O <= 64 ? 64 : 128;
    const int bic = dc_tile_features_for(I, d);
    const int64_t tiles_i = (I + bic - 1) / bic;
    const OutTiling ot = out_tiling(I, O, d);
    // a streamed tail is no tile of the matrix-core launch
    const int64_t tiles = tiles_i * (p.bn == 128 && ot.tail_kind == 2 ? ot.wide_tiles : (O + p.bn - 1) / p.bn);
    const bool mixed = p.bn == 128 && ot.tail_kind == 1;
    // at least 256 rows per slice; a small batch with few tiles may go down to one 32-row chunk per
    // workgroup, which shortens the serial chain of chunks when only a handful of workgroups exist
    const int64_t min_rows = (tiles < 64 && B < 4096 && !(test_hooks() & TEST_DC_MIN_256_ROWS)) ? 32 : 256;
    int64_t max_s = (B + min_rows - 1) / min_rows;
    const int64_t bytes_per_slice = (int64_t)I * K * O * 4;
    const int64_t max_by_bytes = ((int64_t)512 << 20) / bytes_per_slice;
    if (max_s > max_by_bytes) max_s = max_by_bytes;
    if (max_s > 1024) max_s = 1024;
    if (max_s < 1) max_s = 1;
    // Estimated cost of a slice count, in units of one tile row of a 128-wide tile: the slice
    // kernel runs ceil(workgroups / 512) rounds of rows_per_slice rows each, and every slice adds
    // one partial tensor that is written once and read once (about 4 TB/s against ~140 ns per row).
    int64_t best = 1;
    double best_cost = -1.0;
    for (int64_t sl = 1; sl <= max_s; ++sl) {
        int64_t r = (B + sl - 1) / sl;
        r = (r + 31) / 32 * 32;
        double kernel;
        if (mixed) {
            // two launches: the 128-wide tiles, then the 64-wide tail tile (about half the time per row)
            kernel = (double)r * ((double)((tiles_i * ot.wide_tiles * sl + 511) / 512) +
                                  0.5 * (double)((tiles_i * sl + 511) / 512));
        } else {
            kernel = (double)((tiles * sl + 511) / 512) * (double)r * (p.bn / 128.0);
        }
        const double partials = (double)sl * (double)bytes_per_slice * 2.0 / 4.0e12 / 140.0e-9;
        // more than one slice needs the slice-sum launch (about 6 us, 40 row units) that a single slice avoids
        const double cost = kernel + partials + (sl > 1 ? 40.0 : 0.0);
        if (best_cost < 0.0 || cost < best_cost * 0.995) { best_cost = cost; best = sl; }
    }
    int64_t rows = (B + best - 1) / best;
    rows = (rows + 31) / 32 * 32;
    if (rows < 32) rows = 32;
    p.rows_per_slice = (int)rows;
    p.slices = (int)((B + rows - 1) / rows);
    if (p.slices < 1) p.slices = 1;
    return p;
}

inline bool pair_eligible(int64_t B, int I_up, int O_up, int I_lo, int d)
{
    if (!degree_specialised(d) || O_up > 64 || O_up <= NARROW_MAX_OUT) return false;
    if (use_narrow_in(B, I_up, O_up, d) || !use_narrow_in(B, I_lo, I_up, d)) return false;
    if (plan_dC(B, I_up, O_up, d).slices < 2) return false;                     // a single slice writes dC itself
    return (int64_t)((O_up + 31) / 32) * I_up <= 512 && (int64_t)((I_up + 31) / 32) * I_lo <= 512;   // sums small enough to share the combine launch
}

// Column blocks per tile: the count (1..4) that covers the I*D columns of G with the
// fewest 32-column MFMA blocks; ties go to the wider tile (more reuse of the dy tile).
inline int dx_column_blocks(int I, int D)
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

// The feature-per-lane kernel works on 32-feature tiles; it is taken for degrees up to 6
// (measured slower at degree 8, where its eight accumulator blocks leave too few registers)
// unless it needs over 30 % more MFMA blocks than the packed-column kernel (very narrow feature
// counts): per block it is the faster of the two by about a fifth (257 and 80 features at degrees 5
// and 3 were measured both ways).
inline bool dx_feature_per_lane(int I, int D)
{
    if (D > 6) return false;
    const int nb = dx_column_blocks(I, D);
    const int64_t packed = (int64_t)((I + 32 * nb / D - 1) / (32 * nb / D)) * nb;
    const int64_t per_lane = (int64_t)((I + 31) / 32) * D;
    return per_lane * 100 <= packed * 130;
}

inline bool shape_fits(int64_t B, int I, int O, int d)
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
constexpr int NARROW_THREADS = 256;
constexpr int NARROW_RB = 8;   // consecutive rows per lane group and step (memory-level parallelism)
constexpr int NARROW_FWD_WGS = 2048, NARROW_BWD_WGS = 512;

inline bool use_narrow(int64_t B, int I, int O, int d)
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
inline NarrowPlan plan_narrow(int64_t B, int I, int target)
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

// Forward contraction split.  With few output tiles (small batch) one workgroup per tile
// leaves most of the chip idle and each workgroup with a very long contraction, so the
// input features are cut into `splits` ranges whose partial outputs a second kernel adds in
// range order (the paper's Partial + Combine scheme of Sec. 4.4, used only where it pays).
struct FwdPlan {
    int splits;            // 1 = no split, no workspace
    int chunks_per_split;  // forward chunks (of forward_chunk_features(d) features) per range
};

inline FwdPlan plan_forward(int64_t B, int I, int O, int d)
{
    const int bi = forward_chunk_features(d);
    const int n_chunks = (I + bi - 1) / bi;
    const int64_t tiles = ((B + 127) / 128) * ((O + (O <= 64 ? 63 : 127)) / (O <= 64 ? 64 : 128));
    FwdPlan p{1, n_chunks};
    if (n_chunks < 4) return p;
    if (tiles >= 256) {
        // Enough tiles, but with a tail tile they come as two launches that may each leave compute
        // units idle (257 outputs at 16000 rows: 250 + 125 workgroups).  Estimated time per range
        // count, in microseconds: both launches, plus writing and summing the partial planes.
        const OutTiling ot = out_tiling(I, O, d);
        const int64_t row_tiles = (B + 127) / 128;
        if (O <= 128 || ot.tail_begin < 0 || row_tiles * ot.wide_tiles >= 384) return p;
        const double tail_tile = ot.tail_kind == 1 ? 0.5 : 0.0;   // a streamed tail is one short launch of its own
        const double t_chunk = 0.1333 * bi * (d + 1);
        int best = 1;
        double best_us = 0.0;
        for (int sp = 1; sp <= 4 && sp <= n_chunks / 2; ++sp) {
            const int len = (n_chunks + sp - 1) / sp;
            double us = t_chunk * len * (launch_rounds(row_tiles * ot.wide_tiles * sp) + tail_tile * launch_rounds(row_tiles * sp));
            if (sp > 1) us += 6.0 + (2.0 * sp + 1.0) * (double)B * O * 4.0 / 3.0e6;
            if (sp == 1 || us < best_us * 0.97) { best_us = us; best = sp; }
        }
        if (best > 1) {
            p.chunks_per_split = (n_chunks + best - 1) / best;
            p.splits = (n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
        }
        return p;
    }
    int64_t want = (512 + tiles - 1) / tiles;
    if (want > n_chunks / 2) want = n_chunks / 2;      // at least 2 chunks per range
    if (want > 64) want = 64;
    if (want < 2) return p;
    p.chunks_per_split = (int)((n_chunks + want - 1) / want);
    p.splits = (n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return p;
}

// The same for the input gradient: its contraction runs over the outputs, in chunks of
// `chunk_outputs`; `feature_tiles` = column tiles of the chosen dx kernel.
inline FwdPlan plan_dx_split(int64_t B, int feature_tiles, int O, int chunk_outputs)
{
    const int n_chunks = (O + chunk_outputs - 1) / chunk_outputs;
    const int64_t tiles = ((B + 127) / 128) * feature_tiles;
    FwdPlan p{1, n_chunks};
    if (tiles >= 256 || n_chunks < 4) return p;
    int64_t want = (512 + tiles - 1) / tiles;
    if (want > n_chunks / 2) want = n_chunks / 2;
    if (want > 32) want = 32;
    if (want < 2) return p;
    p.chunks_per_split = (int)((n_chunks + want - 1) / want);
    p.splits = (n_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return p;
}

// dx kernel choice and its split, in one place for the launch code and the workspace query
struct DxPlan {
    bool per_lane;     // feature-per-lane kernel (else packed columns)
    int nb;            // column blocks of the packed kernel
    int feature_tiles;
    FwdPlan split;
    // A feature count just above a multiple of 32 (257): the feature-per-lane launch covers features
    // [0, tail_begin) in full tiles and a second, packed-column launch with tail_nb column blocks the
    // few features from tail_begin on, instead of one 32-feature tile that is nearly all padding.
    // tail_begin = I: no second launch.
    int tail_begin;
    int tail_nb;
    int tail_tiles;
};

inline DxPlan plan_dx(int64_t B, int I, int O, int d)
{
    DxPlan p;
    p.per_lane = d >= 1 && dx_feature_per_lane(I, d);
    p.nb = d >= 1 ? dx_column_blocks(I, d) : 1;
    p.tail_begin = I;
    p.tail_nb = 1;
    p.tail_tiles = 0;
    if (p.per_lane) {
        p.feature_tiles = (I + 31) / 32;
        p.split = plan_dx_split(B, p.feature_tiles, O, d <= 4 ? 32 : 16);
        // second launch for the remainder: only unsplit contractions (both launches write dx itself),
        // at least two full tiles, and a remainder that fits one packed tile of at most two column blocks
        const int rem = I % 32;
        const bool pays = B * (int64_t)O >= ((int64_t)1 << 21) || (test_hooks() & TEST_DX_TAIL_ANY_SIZE);   // enough work for a launch
        if (rem > 0 && I >= 64 && p.split.splits == 1 && pays) {
            const int nb = rem * d <= 32 ? 1 : (rem * d <= 64 ? 2 : 0);
            if (nb > 0 && nb * 3 <= d) {   // the tail's column blocks (slower per block) against the d blocks of a padded tile
                p.tail_begin = I - rem;
                p.tail_nb = nb;
                p.tail_tiles = 1;
                p.feature_tiles = I / 32;
            }
        }
    } else {
        const int bix = 32 * p.nb / (d >= 1 ? d : 1);
        p.feature_tiles = (I + bix - 1) / bix;
        p.split = plan_dx_split(B, p.feature_tiles, O, 32);
    }
    return p;
}

}  // namespace chebykan
