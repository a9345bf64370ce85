// Selection among the compiled variants of the dither + sign + pack kernel (included by fo_enc.hip, which
// instantiates the variants without the diagnostic counters, and by fo_enc_stats.hip, which instantiates those with).
#pragma once
#include "fo_host.h"

namespace fo_host {

// The packing kernels are compiled per (dither on/off, transform length below 256).
template <int IN, bool STATS>
int launch_pack_s(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    const bool dither = c.dither == FO_DITHER_UNIFORM, small = c.S < 8;
    const dim3 block(kThreads);
    if (c.K > 1) { // the K-fold quantiser of the server's message
        if (dither && small) return launch(pl, kid, k_contig<IN, OUT_PACK, true, true, 0, true, STATS>, grid, block, st, c, tab);
        if (dither) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 0, true, STATS>, grid, block, st, c, tab);
        return launch(pl, kid, k_contig<IN, OUT_PACK, false, false, 0, true, STATS>, grid, block, st, c, tab);
    }
    if (dither && c.S == 15) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 15, false, STATS>, grid, block, st, c, tab);
    if constexpr (IN == IN_GRAD && !STATS) {
        // block lengths of the blocked workload, compiled for their stage count; tiles that lie inside the input
        // whole go to a variant without the per-chunk end-of-input checks
        if (dither && (c.S == 10 || c.S == 12 || c.S == 14)) {
            const uint64_t full64 = c.len_in >> kTileLog2;
            const uint32_t nfull = (uint32_t)(full64 < grid.x ? full64 : grid.x);
            ContigArgs cc = c;
            auto go = [&](auto sc, auto guarded, uint32_t tile0, uint32_t ntile) -> int {
                cc.tile0 = tile0;
                return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, decltype(sc)::value, false, false, decltype(guarded)::value>,
                              dim3(ntile, grid.y), block, st, cc, tab);
            };
            auto both = [&](auto sc) -> int {
                if (nfull) FO_TRY(go(sc, std::false_type{}, 0u, nfull));
                if (nfull < grid.x) FO_TRY(go(sc, std::true_type{}, nfull, grid.x - nfull));
                return FO_OK;
            };
            if (c.S == 10) return both(std::integral_constant<int, 10>{});
            if (c.S == 12) return both(std::integral_constant<int, 12>{});
            return both(std::integral_constant<int, 14>{});
        }
    }
    if (dither && small) return launch(pl, kid, k_contig<IN, OUT_PACK, true, true, 0, false, STATS>, grid, block, st, c, tab);
    if (dither) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 0, false, STATS>, grid, block, st, c, tab);
    return launch(pl, kid, k_contig<IN, OUT_PACK, false, false, 0, false, STATS>, grid, block, st, c, tab);
}

} // namespace fo_host
