// Host build of the workgroup -> work item -> tile map and of the split plan, for tests/test_tile_map_host.py.
// Compiled for the host only; nothing here touches a GPU.
#include "../paper_2605_19269_amd/csrc/gemm_kernel.hpp"
#include "../paper_2605_19269_amd/csrc/splitk_plan.hpp"

extern "C" {

// plan[0..4] = first shared tile, shared tiles, chunks, exchange slots per shared tile, pieces per range; returns the
// workspace bytes
__attribute__((visibility("default"))) size_t host_plan(int64_t M, int64_t N, int64_t K, int f8, int *plan)
{
    const coda::SplitPlan pl = coda::plan_splitk(M, N, K, f8 != 0);
    plan[0] = pl.first; plan[1] = pl.tail; plan[2] = pl.chunks; plan[3] = pl.stride; plan[4] = pl.pieces;
    return coda::splitk_bytes(pl);
}

// out[8 * bid ..] = tile row, tile column, part, parts, first K-step, K-steps, slot, tile id of the work item of
// workgroup bid (K-steps = 0: a workgroup that leaves at once)
__attribute__((visibility("default"))) void host_tile_map(int tiles_m, int tiles_n, int first, int tail, int chunks, int kt_all, int nwg,
                                                          int *out)
{
    for (int bid = 0; bid < nwg; ++bid) {
        const coda::WorkItem w = coda::locate_block(first, tail, chunks, bid, kt_all);
        int tm = -1, tn = -1;
        if (w.kcnt > 0 || bid < first || chunks == 0) coda::tile_coords(w.tile, tiles_m * tiles_n, tiles_m, tiles_n, tm, tn);
        int *o = out + 8 * bid;
        o[0] = tm; o[1] = tn; o[2] = w.split; o[3] = w.nsplit; o[4] = w.kbeg; o[5] = w.kcnt; o[6] = w.slot; o[7] = w.tile;
    }
}

}
