// splitk_plan.hpp -- host-side plan of the split-K launches (which tiles are shared, by how many workgroups, and the
// workspace that takes).  Pure host arithmetic, shared by the C ABI and by the host tests of the workgroup -> tile map.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace coda {

constexpr int64_t PLAN_TILE_M = 256, PLAN_TILE_N = 256;   // the kernels' workgroup tile (checked against the kernel config where both are seen)

// Split-K plan (tiles and K-steps counted with their ragged edges).  Two cases:
//  * few tiles: at most 64 output tiles leave at least three quarters of the 256 compute units without one (measured:
//    with 64 tiles 4 parts win 1.4x, with 128 tiles 2 parts lose to the exchange of partial tiles): every tile is shared;
//  * partly filled last round: more than 256 tiles whose count is not a multiple of 256 and whose remainder fills at
//    most half of the chip: only the tiles of that last round are shared, so that it takes 1/parts of a round.  Worth
//    it when the contraction length a workgroup is spared clearly outweighs the exchange (about 35 us, the time of ~1400
//    contraction elements of a bf16 tile; the partly filled round itself runs faster than a full one): measured +16 % at
//    320 tiles and +2 % at 384 tiles with K = 8192, +5 % at 320 tiles with K = 4096.
// Every part gets at least 32 K-steps of 32 bf16 (64 fp8) elements and an even number of K-steps.
constexpr int64_t SPLITK_CUS = 256, SPLITK_MAX = 8, SPLITK_MIN_K = 1024, SPLITK_MAX_TILES = 64, SPLITK_TAIL_MIN_SPARED = 3072;
struct SplitPlan {
    int parts;    // <= 1: no split
    int first;    // tiles with id >= first are shared by `parts` workgroups each
    int shared;   // number of shared tiles
};
inline SplitPlan plan_splitk(int64_t M, int64_t N, int64_t K, bool f8 = false)
{
    const SplitPlan none = {1, 0, 0};
    if (M <= 0 || N <= 0 || K <= 0) return none;
    const int64_t tiles = ((M + PLAN_TILE_M - 1) / PLAN_TILE_M) * ((N + PLAN_TILE_N - 1) / PLAN_TILE_N);
    const int64_t scale = f8 ? 2 : 1;                         // an fp8 K-step covers twice the elements in the same time
    const int64_t steps = (K + scale * 64 - 1) / (scale * 64) * 2;   // K-steps of 32 bf16 / 64 fp8 elements, in whole pairs
    auto fit = [&](int64_t s) {
        if (s > K / (scale * SPLITK_MIN_K)) s = K / (scale * SPLITK_MIN_K);
        if (s > SPLITK_MAX) s = SPLITK_MAX;
        // the kernels walk their K-steps in pairs: every part must get an even number
        while (s >= 2 && steps % (2 * s)) --s;
        return s >= 2 ? s : (int64_t)1;
    };
    if (tiles <= SPLITK_MAX_TILES) {
        const int64_t s = fit(SPLITK_CUS / tiles);
        return s >= 2 ? SplitPlan{(int)s, 0, (int)tiles} : none;
    }
    const int64_t rem = tiles % SPLITK_CUS;
    if (tiles < SPLITK_CUS || rem == 0 || rem > SPLITK_CUS / 2) return none;
    const int64_t s = fit(SPLITK_CUS / rem);
    if (s < 2 || K - K / s < scale * SPLITK_TAIL_MIN_SPARED) return none;
    return SplitPlan{(int)s, (int)(tiles - rem), (int)rem};
}
constexpr size_t SPLITK_CNT_BYTES = 1024;   // ticket counters (at most 128 shared tiles x 4 bytes), kept apart from the partials
inline size_t splitk_bytes(const SplitPlan &pl)
{
    if (pl.parts <= 1) return 0;
    return SPLITK_CNT_BYTES + (size_t)pl.shared * (size_t)pl.parts * PLAN_TILE_M * PLAN_TILE_N * sizeof(float);
}


}  // namespace coda
