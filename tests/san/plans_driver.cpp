// Host-only driver of the library's planning code (csrc/plans.h), built with
// -fsanitize=address,undefined by tests/test_sanitizers_host.py.  It sweeps seeded random and
// extreme shapes through every plan function and checks the invariants the launch code relies
// on; any violation (or any sanitizer report) ends the run with a non-zero status.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <initializer_list>

#include "../../paper_2511_14852_amd/csrc/plans.h"

using namespace chebykan;

static int failures = 0;
#define CHECK(cond, ...)                                   \
    do {                                                   \
        if (!(cond)) {                                     \
            fprintf(stderr, "violated: %s  (", #cond);    \
            fprintf(stderr, __VA_ARGS__);                  \
            fprintf(stderr, ")\n");                        \
            if (++failures > 20) exit(1);                  \
        }                                                  \
    } while (0)

static uint64_t state = 251114852ull;
static uint64_t next_u64()
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;   // a plain 64-bit LCG: any seeded stream will do
    return state >> 11;
}
static int64_t pick(int64_t lo, int64_t hi) { return lo + (int64_t)(next_u64() % (uint64_t)(hi - lo + 1)); }

static void check_shape(int64_t B, int I, int O, int d)
{
    const int K = d + 1;
    const OutTiling ot = out_tiling(I, O, d);
    CHECK(ot.wide_tiles >= 0 && (ot.tail_begin < 0 || (ot.tail_begin % 128 == 0 && O - ot.tail_begin >= 1 && O - ot.tail_begin <= 64)),
          "O=%d", O);
    CHECK((ot.tail_kind == 0) == (ot.tail_begin < 0), "O=%d kind=%d", O, ot.tail_kind);
    CHECK(ot.tail_kind != 2 || (O - ot.tail_begin <= NARROW_MAX_OUT && (int64_t)I * (O - ot.tail_begin) * K <= 16384), "O=%d I=%d", O, I);
    CHECK((int64_t)ot.wide_tiles * 128 + (ot.tail_kind == 1 ? 64 : ot.tail_kind == 2 ? O - ot.tail_begin : 0) >= O, "O=%d", O);

    const DcPlan dc = plan_dC(B, I, O, d);
    CHECK(dc.bn == 64 || dc.bn == 128, "bn=%d", dc.bn);
    CHECK(dc.slices >= 1 && dc.rows_per_slice >= 32 && dc.rows_per_slice % 32 == 0, "B=%lld I=%d O=%d d=%d slices=%d rows=%d",
          (long long)B, I, O, d, dc.slices, dc.rows_per_slice);
    CHECK((int64_t)dc.slices * dc.rows_per_slice >= B, "rows covered: B=%lld slices=%d rows=%d", (long long)B, dc.slices, dc.rows_per_slice);
    CHECK((int64_t)(dc.slices - 1) * dc.rows_per_slice < (B > 0 ? B : 1), "no empty trailing slice: B=%lld slices=%d rows=%d",
          (long long)B, dc.slices, dc.rows_per_slice);
    CHECK((int64_t)dc.slices * I * K * O * 4 <= ((int64_t)513 << 20) || dc.slices == 1, "partial buffers capped: %d slices", dc.slices);
    const int bic = dc_tile_features_for(I, d);
    CHECK(bic >= 1 && bic * K <= 128, "bic=%d K=%d", bic, K);

    const FwdPlan fp = plan_forward(B, I, O, d);
    const int bi = forward_chunk_features(d);
    const int n_chunks = (I + bi - 1) / bi;
    CHECK(bi >= 2 && bi % 2 == 0, "bi=%d", bi);
    CHECK(fp.splits >= 1 && fp.chunks_per_split >= 1, "splits=%d", fp.splits);
    CHECK((int64_t)fp.splits * fp.chunks_per_split >= n_chunks && (int64_t)(fp.splits - 1) * fp.chunks_per_split < n_chunks,
          "forward ranges cover the chunks exactly: I=%d d=%d splits=%d per=%d", I, d, fp.splits, fp.chunks_per_split);

    if (d >= 1) {
        const DxPlan dx = plan_dx(B, I, O, d);
        CHECK(dx.nb >= 1 && dx.nb <= 4 && dx.feature_tiles >= 1, "nb=%d tiles=%d", dx.nb, dx.feature_tiles);
        const int feats = dx.per_lane ? 32 : 32 * dx.nb / d;
        CHECK(dx.tail_begin >= 0 && dx.tail_begin <= I, "tail_begin=%d I=%d", dx.tail_begin, I);
        CHECK(feats >= 1 && (int64_t)dx.feature_tiles * feats >= dx.tail_begin, "dx tiles cover the features: I=%d d=%d", I, d);
        if (dx.tail_begin < I) {
            // second launch: packed columns over the features past the full 32-feature tiles, contraction unsplit
            CHECK(dx.per_lane && dx.split.splits == 1 && dx.tail_begin % 32 == 0 && dx.tail_begin >= 32, "tail_begin=%d", dx.tail_begin);
            CHECK((dx.tail_nb == 1 || dx.tail_nb == 2) && dx.tail_tiles >= 1, "tail_nb=%d tiles=%d", dx.tail_nb, dx.tail_tiles);
            CHECK((int64_t)dx.tail_tiles * (32 * dx.tail_nb / d) >= I - dx.tail_begin, "tail tiles cover the rest: I=%d d=%d", I, d);
            CHECK((int64_t)dx.feature_tiles * 32 == dx.tail_begin, "full tiles end where the tail begins (I=%d)", I);
        }
        const int co = dx.per_lane ? (d <= 4 ? 32 : 16) : 32;
        const int nco = (O + co - 1) / co;
        CHECK((int64_t)dx.split.splits * dx.split.chunks_per_split >= nco &&
                  (int64_t)(dx.split.splits - 1) * dx.split.chunks_per_split < nco,
              "dx ranges cover the output chunks exactly: O=%d splits=%d per=%d", O, dx.split.splits, dx.split.chunks_per_split);
        CHECK(!dx.per_lane || d <= 6, "feature-per-lane kernel exists up to degree 6 (d=%d)", d);
    }

    if (O <= NARROW_MAX_OUT) {
        for (int target : {NARROW_FWD_WGS, NARROW_BWD_WGS}) {
            const NarrowPlan np = plan_narrow(B, I, target);
            CHECK(np.G >= 8 && np.G <= 64 && (np.G & (np.G - 1)) == 0, "G=%d", np.G);
            CHECK(np.rows_per_wg % (NARROW_RB * (NARROW_THREADS / np.G)) == 0 && np.rows_per_wg > 0, "rows_per_wg=%d G=%d", np.rows_per_wg, np.G);
            CHECK((int64_t)np.slices * np.rows_per_wg >= B, "narrow rows covered: B=%lld", (long long)B);
        }
    }
    if (use_narrow_in(B, I, O, d)) {
        const NarrowInPlan ni = plan_narrow_in(B);
        CHECK(ni.rows_per_slice % 32 == 0 && ni.rows_per_slice >= 128 && (int64_t)ni.slices * ni.rows_per_slice >= B,
              "few-inputs plan: B=%lld slices=%d rows=%d", (long long)B, ni.slices, ni.rows_per_slice);
        CHECK(I * K <= 64 && O <= 64, "few-inputs tile: I=%d K=%d O=%d", I, K, O);
    }
    (void)shape_fits(B, I, O, d);
    (void)launch_rounds(B);
}

int main()
{
    const int degrees[] = {0, 1, 2, 3, 4, 5, 6, 7, 8, 15, 24, 32};
    // the benchmark configurations and the extremes the entry points accept
    const int64_t fixed[][4] = {{256, 64, 64, 4}, {65536, 8, 64, 6}, {65536, 64, 64, 6}, {65536, 64, 1, 6}, {32768, 80, 512, 3},
                                {32768, 512, 512, 3}, {32768, 512, 256, 3}, {16000, 257, 512, 5}, {16000, 512, 257, 5},
                                {16384, 1024, 1024, 8}, {128, 40, 256, 8}, {64, 256, 512, 15}, {32, 512, 1024, 24},
                                {1, 1, 1, 0}, {1, 1, 1, 32}, {2147483647LL, 1, 1, 6}, {2147483647LL, 8, 64, 6}, {1, 65535, 1, 1},
                                {1, 1, 65535, 1}, {7, 65535, 8190, 3}, {16777293, 8, 64, 6}, {16777221, 64, 1, 6}};
    for (const auto& f : fixed) check_shape(f[0], (int)f[1], (int)f[2], (int)f[3]);
    for (int rep = 0; rep < 200000; ++rep) {
        const int d = degrees[pick(0, (int)(sizeof(degrees) / sizeof(degrees[0])) - 1)];
        const int64_t B = rep % 3 == 0 ? pick(1, 300) : rep % 3 == 1 ? pick(1, 70000) : pick(1, 40000000);
        int I = (int)(rep % 2 ? pick(1, 80) : pick(1, 2100));
        int O = (int)(rep % 5 == 0 ? pick(1, 4) : rep % 5 < 3 ? pick(1, 140) : pick(1, 2100));
        if ((int64_t)I * O * (d + 1) > ((int64_t)1 << 31) - 1) continue;
        check_shape(B, I, O, d);
    }
    if (failures) { fprintf(stderr, "%d violations\n", failures); return 1; }
    printf("plans: all invariants hold\n");
    return 0;
}
