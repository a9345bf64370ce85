// Launch sequences of the server (Sec. 4, "Server-to-workers"): decode every message, average, re-encode.
#include "fo_host.h"
#include "fo_server_high.h"

namespace fo_host {

int launch_server(fo_plan *pl, const uint64_t *bits_up, const float *scales_up, uint64_t round, uint64_t *bits_down,
                  float *scales_down, float *gbar_or_null, hipStream_t st)
{
    const Rng r = rng_of(pl, round);
    const uint32_t M = pl->p.M;
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    // server amplitude: the theorem's rule from the workers' amplitudes now, or from the norm of the mean later
    const bool l2s = pl->p.server_scale == FO_SERVER_SCALE_L2;
    if (!l2s)
        FO_TRY(launch_server_scales(pl, st, scales_up, scales_down));
    auto finalize_server_scales = [&]() -> int { // after a fused strided pass that left the tile sums of squares of gbar
        return launch_finalize_scales(pl, st, 1, pl->coef_lambda_s, scales_down, 0);
    };
    const float mean_coef = pl->rsqrtb / (float)M;
    const bool zero_transform = pl->p.eps_mode == FO_EPS_SHARED_ALL;
    if (zero_transform) {
        // the server shares the workers' eps: its pre-quantisation vector is (lambda / M)(2 c - M), no transform
        ShallArgs z;
        z.bits_up = bits_up; z.dst = bits_down; z.lam = scales_up; z.lam_s = scales_down;
        z.W = pl->W; z.logb = pl->logb; z.M = M; z.K = pl->p.K; z.planes = pl->planes; z.dither = pl->p.dither;
        z.k0 = r.k0; z.k1 = r.k1; z.round_lo = r.round_lo; z.round_dev = r.round_dev; z.sqrtb = pl->sqrtb;
        if (l2s) { // lambda^s from ||gbar||: an exact integer count first
            const dim3 bg((unsigned)((pl->nblocks + 255) / 256));
            FO_TRY(launch(pl, KID_SCALES, k_zero_u64, bg, dim3(256), st, pl->blk_sums, pl->nblocks));
            FO_TRY(launch(pl, KID_SHALL, k_shall_sumsq, dim3((unsigned)((pl->W + 15) / 16)), dim3(256), st, z, pl->blk_sums));
            FO_TRY(launch(pl, KID_SCALES, k_shall_scales, bg, dim3(256), st, pl->blk_sums, scales_up, pl->nblocks, M,
                          pl->coef_lambda_s, scales_down));
        }
        FO_TRY(launch(pl, KID_SHALL, k_shall, dim3((unsigned)((pl->W + 15) / 16)), dim3(256), st, z));
        if (!gbar_or_null) return FO_OK;
        // the mean itself was asked for (checking): one inverse transform of the summed sign vectors, below
    }
    if (pl->p.eps_mode != FO_EPS_INDEPENDENT && pl->npass == 2) {
        // the same for three-pass transforms (blocks above 2^25): counts -> low stages (int32) -> middle stages -> the
        // shared pass on the top stages (amplitude, eps, eps^s, forward top stages) -> middle stages forward -> low pass
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W; c.M = M;
        c.scales = const_cast<float *>(scales_up); c.scales_stride = 0;
        c.party0 = 0; c.eps_party0 = kPartyAllWorkers;
        c.dst = pl->buf_a; c.dst_stride = 0;
        const dim3 grid1((unsigned)pl->ntiles, 1), block(kThreads);
        FO_TRY(launch(pl, KID_COUNT_LOW, (k_contig<IN_COUNT, OUT_I32, false, false, 15>), grid1, block, st, c, none));
        StridedArgs s0 = strided_base(pl, r, 0);
        s0.src = pl->buf_a; s0.dst = pl->buf_c;
        FO_TRY(launch_strided<SM_MID_I32>(pl, KID_DEC_MID, grid1, st, s0, none));
        StridedArgs s = strided_base(pl, r, 1);
        s.src = pl->buf_c; s.dst = pl->buf_b;
        s.scales = scales_up; s.scales_stride = 0;
        s.gbar = gbar_or_null;
        s.out_coef = mean_coef; s.eps_party0 = FO_PARTY_SERVER;
        s.partials = l2s ? pl->partials : nullptr;
        FO_TRY(launch_strided<SM_SHARED>(pl, KID_SERVER_HIGH, grid1, st, s, none));
        if (zero_transform) return FO_OK;
        if (l2s) FO_TRY(finalize_server_scales());
        StridedArgs s2 = strided_base(pl, r, 0);
        s2.src = pl->buf_b; s2.dst = pl->buf_c;
        FO_TRY(launch_strided<SM_MID_F32>(pl, KID_ENC_MID, grid1, st, s2, none));
        ContigArgs e = contig_base(pl, r);
        e.src = pl->buf_c; e.dst = bits_down;
        e.scales = scales_down;
        e.party0 = FO_PARTY_SERVER; e.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(e, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid1, st, e, none));
        return FO_OK;
    }
    if (pl->p.eps_mode != FO_EPS_INDEPENDENT && pl->npass <= 1) {
        // one eps and one amplitude for all workers: sum the packed sign vectors per coordinate (vertical
        // popcount), then a single inverse transform instead of M
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W; c.M = M;
        c.scales = const_cast<float *>(scales_up); c.scales_stride = 0; // worker 0's amplitudes are everybody's
        c.party0 = 0; c.eps_party0 = kPartyAllWorkers;
        const dim3 grid1((unsigned)pl->ntiles, 1), block(kThreads);
        if (pl->npass == 0) {
            float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
            c.dst = gbar; c.len_out = pl->ntot; c.store_mode = STORE_SET; c.out_coef = mean_coef;
            FO_TRY(launch(pl, KID_COUNT_LOW, (k_contig<IN_COUNT, OUT_F32>), grid1, block, st, c, none));
            if (zero_transform) return FO_OK;
            return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down,
                                 0, nullptr, 0, st);
        }
        c.dst = pl->buf_a; c.dst_stride = 0;
        FO_TRY(launch(pl, KID_COUNT_LOW, (k_contig<IN_COUNT, OUT_I32, false, false, 15>), grid1, block, st, c, none));
        StridedArgs s = strided_base(pl, r, 0);
        s.src = pl->buf_a; s.dst = pl->buf_b;
        s.scales = scales_up; s.scales_stride = 0;
        s.gbar = gbar_or_null;
        s.out_coef = mean_coef; s.eps_party0 = FO_PARTY_SERVER;
        s.partials = l2s ? pl->partials : nullptr;
        s.dst_pad = pl->pad32;
        FO_TRY(launch_strided<SM_SHARED>(pl, KID_SERVER_HIGH, grid1, st, s, none));
        if (zero_transform) return FO_OK;
        if (l2s) FO_TRY(finalize_server_scales());
        ContigArgs e = contig_base(pl, r);
        e.src = pl->buf_b; e.dst = bits_down; e.src_pad = pl->pad32;
        e.scales = scales_down;
        e.party0 = FO_PARTY_SERVER; e.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(e, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid1, st, e, none));
        return FO_OK;
    }
    if (pl->npass == 0) {
        // the transform fits a tile: the mean tile by tile in registers, then the ordinary encode
        float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
        ServerTileArgs sa;
        sa.enc = contig_base(pl, r);
        sa.enc.src = gbar;
        sa.bits_up = bits_up; sa.scales_up = scales_up; sa.M = M;
        sa.coef = 2.f * mean_coef; // the decode side carries half values
        // one workgroup fills a compute unit (its two exchange buffers take most of the LDS) and walks over tiles
        const unsigned nwg = (unsigned)(pl->ntiles < pl->num_cus ? pl->ntiles : pl->num_cus);
        FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_mfma, dim3(nwg), dim3(kMfThreads), st, sa, (uint32_t)pl->ntiles));
        return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down, 0,
                             nullptr, 0, st);
    }
    if (pl->logb == 16) {
        // blocks of exactly two tiles: the mean in one pass over the packed signs, two workgroups per block, then the
        // one-pass encode of blocks of that length
        float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
        ServerTileArgs sa;
        sa.enc = contig_base(pl, r);
        sa.enc.src = gbar;
        sa.bits_up = bits_up; sa.scales_up = scales_up; sa.M = M;
        sa.coef = 2.f * mean_coef; // the decode side carries half values
        const uint32_t nunits = (uint32_t)(2 * pl->nblocks);
        const unsigned nwg = nunits < pl->num_cus ? nunits : pl->num_cus;
        FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_mfma_pair, dim3(nwg), dim3(kMfThreads), st, sa, nunits));
        return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down, 0,
                             pl->buf_a, 0, st);
    }
    if (pl->npass == 2) {
        // three-pass transforms (blocks above 2^25): low stages of all workers (bits -> int32), the middle stages in
        // place, one fused pass on the top stages that forms the mean and starts the re-encode, the middle stages
        // forward, the low pass that dithers and packs
        const dim3 gridM((unsigned)pl->ntiles, M), grid1((unsigned)pl->ntiles, 1), block(kThreads);
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W;
        c.dst = pl->buf_a; c.dst_stride = pl->ntot;
        FO_TRY(launch(pl, KID_DEC_LOW, (k_contig<IN_BITS, OUT_I32, false, false, 15>), gridM, block, st, c, none));
        StridedArgs s0 = strided_base(pl, r, 0);
        s0.src = pl->buf_a; s0.src_stride = pl->ntot;
        s0.dst = pl->buf_a; s0.dst_stride = pl->ntot; // in place: a workgroup reads its whole tile before it writes it
        FO_TRY(launch_strided<SM_MID_I32>(pl, KID_DEC_MID, gridM, st, s0, none));
        StridedArgs s = strided_base(pl, r, 1);
        s.src = pl->buf_a; s.src_stride = pl->ntot;
        s.dst = pl->buf_b;
        s.scales = scales_up; s.scales_stride = pl->nblocks;
        s.gbar = gbar_or_null;
        s.M = M; s.out_coef = 2.f * mean_coef; s.eps_party0 = FO_PARTY_SERVER; // the decode side carries half values
        s.partials = l2s ? pl->partials : nullptr;
        FO_TRY((launch_strided<SM_SERVER, false>(pl, KID_SERVER_HIGH, grid1, st, s, none)));
        if (l2s) FO_TRY(finalize_server_scales());
        StridedArgs s2 = strided_base(pl, r, 0);
        s2.src = pl->buf_b; s2.dst = pl->buf_c;
        FO_TRY(launch_strided<SM_MID_F32>(pl, KID_ENC_MID, grid1, st, s2, none));
        ContigArgs e = contig_base(pl, r);
        e.src = pl->buf_c; e.dst = bits_down;
        e.scales = scales_down;
        e.party0 = FO_PARTY_SERVER; e.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(e, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid1, st, e, none));
        return FO_OK;
    }
    // two-pass transforms: M low-stage passes (bits -> int32), one fused high-stage pass that forms the mean
    // and starts the re-encode, one low-stage pass that dithers and packs
    {
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W;
        c.dst = pl->buf_a; c.dst_stride = pl->ntot + pl->ntiles * pl->pad16; c.dst_pad = pl->pad16;
        FO_TRY(launch_declow(pl, dim3((unsigned)pl->ntiles, M), st, c));
    }
    {
        StridedArgs s = strided_base(pl, r, 0);
        s.src = pl->buf_a; s.src_stride = pl->ntot + pl->ntiles * pl->pad16; s.src_pad = pl->pad16;
        s.dst = pl->buf_b; s.dst_pad = pl->pad32;
        s.scales = scales_up; s.scales_stride = pl->nblocks;
        s.gbar = gbar_or_null;
        s.M = M; s.out_coef = 2.f * mean_coef; s.eps_party0 = FO_PARTY_SERVER; // int16 input holds half values
        s.partials = l2s ? pl->partials : nullptr;
        if (s.hb == 10 && pl->server_mfma) // blocks of 2^25: the inverse stages on the matrix cores
            FO_TRY(launch(pl, KID_SERVER_MFMA, k_server_mfma, dim3((unsigned)pl->ntiles), dim3(1024), st, s));
        else
            FO_TRY((launch_strided<SM_SERVER, true>(pl, KID_SERVER_HIGH, dim3((unsigned)pl->ntiles, 1), st, s, none)));
        if (l2s) FO_TRY(finalize_server_scales());
    }
    {
        ContigArgs c = contig_base(pl, r);
        c.src = pl->buf_b; c.src_stride = 0; c.src_pad = pl->pad32;
        c.dst = bits_down; c.dst_stride = 0;
        c.scales = scales_down; c.scales_stride = 0;
        c.party0 = FO_PARTY_SERVER; c.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(c, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, dim3((unsigned)pl->ntiles, 1), st, c, none));
    }
    return FO_OK;
}


} // namespace fo_host
