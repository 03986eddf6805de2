// splitk_plan.hpp -- host-side plan of the split-K launches (which tiles are shared, by how many workgroups, and the
// workspace that takes).  Pure host arithmetic, shared by the C ABI and by the host tests of the workgroup -> tile map.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace coda {

constexpr int64_t PLAN_TILE_M = 256, PLAN_TILE_N = 256;   // the kernels' workgroup tile (checked against the kernel config where both are seen)

// Plan of the shared tiles (tiles and K-steps counted with their ragged edges).  The tiles that would leave compute units
// idle -- all of them when there are fewer than 256, else those of the last, partly filled round of 256 -- form the
// "tail"; its K-steps, laid end to end, are cut into `chunks` equal contiguous ranges, one workgroup each, so that the
// tail takes tail / chunks of a tile time instead of a whole one:
//  * chunks = min(256, tail * parts), parts = min(8, K / 1024): every range gets at least 1024 contraction elements
//    (32 K-steps of 32 bf16, 16 of 64 fp8 elements).  When tail * parts fits the chip every tile is cut into `parts`
//    equal parts; otherwise the 256 ranges straddle tile boundaries (a balanced "stream-K" round);
//  * only when it pays against the exchange of partial tiles through the workspace (256 KB per part, written once and
//    read once: the full-chip exchange costs about 70 us): a workgroup must be spared at least SPLITK_MIN_SPARED_STEPS
//    K-steps of a tile, and must be left with at most SPLITK_MAX_SHARE_NUM / _DEN of one.
// Measured (residual + sum-of-squares program, bf16, against the same launch without workspace): K = 8192: 4 tiles
// 2.7x, 16 tiles 2.4x, 40 tiles +73 %, 64 tiles 1.7x, 72 tiles +18 %, 96 tiles +31 %, 128 tiles +23 %; 272 tiles +36 %,
// 320 tiles +20 %, 384 tiles +10 %, 576 tiles +13 %; K = 4096: 16 tiles +78 %, 64 tiles +21 %, 128 tiles +6 %, 320 tiles
// +8 %, 384 tiles +4 %; K = 2048 (32 K-steps spared at best): 16 tiles +1 to +6 %, 64 tiles -2 %, 384 tiles -9 %.  Rounds
// that are more than half full lose -- 144 tiles -17 %, 160 tiles +0 %, 192 tiles -3 %, 208 tiles -29 % (ranges of 13/16 of
// a tile leave slivers of 1/16, each with its own pipeline fill and exchange), 448 tiles -5 % at K = 8192 and -2 % at
// K = 16384, 496 tiles -19 % -- and run unsplit.  Hence: spared >= 64 K-steps, share <= 1/2 (a round of up to 128 tiles;
// ranges straddle tile boundaries when tail * parts exceeds the chip, e.g. 40 tiles x 8 parts: +73 %).
constexpr int64_t SPLITK_CUS = 256, SPLITK_MAX_PARTS = 8, SPLITK_MIN_K = 1024, SPLITK_MIN_SPARED_STEPS = 64;
constexpr int64_t SPLITK_MAX_SHARE_NUM = 1, SPLITK_MAX_SHARE_DEN = 2;
struct SplitPlan {
    int first;    // tiles below `first` run whole
    int tail;     // number of shared tiles (ids first .. first + tail - 1)
    int chunks;   // workgroups that share them; 0: nothing is shared
    int stride;   // exchange slots per shared tile: the largest number of ranges that reach into one tile
    int pieces;   // 1: every range lies in one tile; 2: ranges straddle tile boundaries (two workgroups per range)
};
inline SplitPlan plan_splitk(int64_t M, int64_t N, int64_t K, bool f8 = false)
{
    const SplitPlan none = {0, 0, 0, 0, 1};
    if (M <= 0 || N <= 0 || K <= 0) return none;
    const int64_t tiles = ((M + PLAN_TILE_M - 1) / PLAN_TILE_M) * ((N + PLAN_TILE_N - 1) / PLAN_TILE_N);
    const int64_t scale = f8 ? 2 : 1;                         // an fp8 K-step covers twice the elements in the same time
    const int64_t pairs = (K + scale * 64 - 1) / (scale * 64);   // pairs of K-steps per tile (K-steps of 32 bf16 / 64 fp8 elements)
    int64_t parts = K / (scale * SPLITK_MIN_K);
    if (parts > SPLITK_MAX_PARTS) parts = SPLITK_MAX_PARTS;
    if (parts < 2) return none;
    const int64_t tail = tiles < SPLITK_CUS ? tiles : tiles % SPLITK_CUS;
    if (tail == 0) return none;
    int64_t chunks = tail * parts < SPLITK_CUS ? tail * parts : SPLITK_CUS;
    if (chunks <= tail) return none;
    // K-steps of the longest range against those of a whole tile
    const int64_t longest = 2 * ((tail * pairs + chunks - 1) / chunks);
    if (2 * pairs - longest < SPLITK_MIN_SPARED_STEPS / (f8 ? 2 : 1)) return none;
    if (SPLITK_MAX_SHARE_DEN * tail > SPLITK_MAX_SHARE_NUM * chunks) return none;
    // ranges per tile: tile a is reached by the ranges that hold its first and its last pair, and those in between
    const int64_t total = tail * pairs;
    int64_t stride = 1;
    for (int64_t a = 0; a < tail; ++a) {
        const int64_t c_lo = ((a * pairs + 1) * chunks + total - 1) / total - 1;
        const int64_t c_hi = (((a + 1) * pairs) * chunks + total - 1) / total - 1;
        if (c_hi - c_lo + 1 > stride) stride = c_hi - c_lo + 1;
    }
    return SplitPlan{(int)(tiles - tail), (int)tail, (int)chunks, (int)stride, chunks % tail == 0 ? 1 : 2};
}
constexpr size_t SPLITK_CNT_BYTES = 1024;   // ticket counters (at most 255 shared tiles x 4 bytes), kept apart from the partials
inline size_t splitk_bytes(const SplitPlan &pl)
{
    if (pl.chunks == 0) return 0;
    return SPLITK_CNT_BYTES + (size_t)pl.tail * (size_t)pl.stride * PLAN_TILE_M * PLAN_TILE_N * sizeof(float);
}

}  // namespace coda
