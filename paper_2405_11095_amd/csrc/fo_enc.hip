// Launch sequences of the encoder (Def. 3.7): single-pass, pair and two- / three-pass geometries.
#include "fo_enc_pack.h"

namespace fo_host {

template int launch_pack_s<IN_GRAD, false>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
template int launch_pack_s<IN_F32, false>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);

namespace {
// Encode of blocks of 2^16 coordinates in one pass.
int launch_pair(fo_plan *pl, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    const bool dither = c.dither == FO_DITHER_UNIFORM;
    const dim3 block(2 * kThreads);
    if (c.K > 1) {
        if (dither) return launch(pl, KID_ENC_PAIR, k_contig_pair<true, true>, grid, block, st, c, tab);
        return launch(pl, KID_ENC_PAIR, k_contig_pair<false, true>, grid, block, st, c, tab);
    }
    if (dither) {
        // blocks that lie inside the input whole: no per-chunk end-of-input checks
        const uint64_t full64 = c.len_in >> 16;
        const uint32_t nfull = (uint32_t)(full64 < grid.x ? full64 : grid.x);
        ContigArgs cc = c;
        if (nfull) FO_TRY(launch(pl, KID_ENC_PAIR, k_contig_pair<true, false, false>, dim3(nfull, grid.y), block, st, cc, tab));
        if (nfull < grid.x) {
            cc.tile0 = 2u * nfull;
            FO_TRY(launch(pl, KID_ENC_PAIR, k_contig_pair<true, false, true>, dim3(grid.x - nfull, grid.y), block, st, cc, tab));
        }
        return FO_OK;
    }
    return launch(pl, KID_ENC_PAIR, k_contig_pair<false, false>, grid, block, st, c, tab);
}

} // namespace

// Encode `nslots` vectors.  Sources: tab (pointer table, nslots entries) or src + slot * src_stride.
// scales_given: scales[] already holds the amplitudes (forced / bound rule); else they come from the
// measured norms.  common: the nslots parties are all the workers of a shared-eps round and must agree
// on one amplitude per block (the largest) before any of them quantises; scales is then [M][nblocks].
int launch_encode(fo_plan *pl, const PtrTab *tab, const float *src, uint64_t src_stride, uint64_t len_in,
                  uint32_t nslots, uint32_t party0, uint64_t round, bool scales_given, uint64_t *bits,
                  uint64_t bits_stride, float *scales, uint64_t scales_stride, float *tmp, uint64_t tmp_stride,
                  hipStream_t st, bool common)
{
    const Rng r = rng_of(pl, round);
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    const PtrTab &tb = tab ? *tab : none;
    const dim3 grid((unsigned)pl->ntiles, nslots), block(kThreads);
    ContigArgs c = contig_base(pl, r);
    c.dst = bits; c.dst_stride = bits_stride;
    c.scales = scales; c.scales_stride = scales_stride;
    c.party0 = party0; c.eps_party0 = eps_party_of(pl, party0);
    set_quantiser(c, pl, party0);
    // amplitude from a measured norm: alpha for a worker, alpha_s for the server's own vector
    const float coef = party0 == FO_PARTY_SERVER ? pl->coef_lambda_s : pl->coef_lambda;
    c.coef_lambda = coef;
    if (pl->npass == 0) {
        c.src = src; c.src_stride = src_stride; c.use_tab = tab ? 1u : 0u;
        c.len_in = len_in;
        c.compute_scale = scales_given ? 0u : 1u;
        if (common && !scales_given) {
            // one extra read of the gradients: norms first, then the common amplitude, then the encode proper
            c.scales_only = 1u;
            FO_TRY(launch_pack<IN_GRAD>(pl, KID_ENC_SINGLE, grid, st, c, tb));
            FO_TRY(launch_common_scales(pl, st, scales, nslots));
            c.scales_only = 0u;
            c.compute_scale = 0u;
        }
        FO_TRY(launch_pack<IN_GRAD>(pl, KID_ENC_SINGLE, grid, st, c, tb));
        return FO_OK;
    }
    if (pl->logb == 16 && !c.stat_clipped) {
        // blocks of exactly two tiles: one pass, a workgroup of 1024 threads per block
        c.src = src; c.src_stride = src_stride; c.use_tab = tab ? 1u : 0u;
        c.len_in = len_in;
        c.compute_scale = scales_given ? 0u : 1u;
        const dim3 pgrid((unsigned)(pl->ntiles / 2), nslots);
        if (common && !scales_given) {
            c.scales_only = 1u;
            FO_TRY(launch_pair(pl, pgrid, st, c, tb));
            FO_TRY(launch_common_scales(pl, st, scales, nslots));
            c.scales_only = 0u;
            c.compute_scale = 0u;
        }
        return launch_pair(pl, pgrid, st, c, tb);
    }
    // transform lengths above 2^15: high stages first (eps flip and norm on load), low stages last
    const uint32_t first = pl->npass - 1;
    StridedArgs s = strided_base(pl, r, first);
    s.src = src; s.src_stride = src_stride; s.use_tab = tab ? 1u : 0u; s.len_in = len_in;
    s.dst = (pl->npass == 2) ? pl->buf_c : tmp; s.dst_stride = (pl->npass == 2) ? 0 : tmp_stride;
    s.partials = pl->partials; s.eps_party0 = eps_party_of(pl, party0);
    // the intermediate in plan scratch has padded rows; the one of fo_encode_noalloc and the server's (tmp == nullptr
    // never happens here) follow the plan's setting as well
    const uint32_t pad = pl->npass == 1 ? pl->pad32 : 0u;
    s.dst_pad = pad;
    if (pl->npass == 2 && nslots != 1) return FO_EINVAL; // three-pass transforms are encoded one party at a time
    FO_TRY(launch_strided<SM_ENC_FIRST>(pl, KID_ENC_HIGH, grid, st, s, tb));
    if (pl->npass == 2) {
        StridedArgs s2 = strided_base(pl, r, 0);
        s2.src = pl->buf_c; s2.dst = tmp; s2.src_stride = 0; s2.dst_stride = tmp_stride;
        FO_TRY(launch_strided<SM_MID_F32>(pl, KID_ENC_MID, grid, st, s2, none));
    }
    if (!scales_given) {
        FO_TRY(launch_finalize_scales(pl, st, nslots, coef, scales, scales_stride));
        if (common) FO_TRY(launch_common_scales(pl, st, scales, nslots));
    }
    c.src = tmp; c.src_stride = tmp_stride;
    c.src_pad = pad;
    FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid, st, c, none));
    return FO_OK;
}


} // namespace fo_host
