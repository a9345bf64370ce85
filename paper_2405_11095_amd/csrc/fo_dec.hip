// Launch sequences of the decoder (Def. 3.8).
#include "fo_host.h"

namespace fo_host {

int launch_declow(fo_plan *pl, dim3 grid, hipStream_t st, const ContigArgs &c)
{
    return launch(pl, KID_DEC_LOW, k_declow, grid, dim3(kThreads), st, c);
}

// Decode one party into out[len_out] with the given store mode.
int launch_decode(fo_plan *pl, const uint64_t *bits, const float *scales, uint64_t round, uint32_t party,
                  float *out, uint64_t len_out, uint32_t store_mode, float out_coef, float delta, float *tmp,
                  hipStream_t st)
{
    const Rng r = rng_of(pl, round);
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    const dim3 grid((unsigned)pl->ntiles, 1), block(kThreads);
    ContigArgs c = contig_base(pl, r);
    c.src = bits; c.src_stride = 0;
    c.scales = const_cast<float *>(scales); c.scales_stride = 0;
    c.party0 = party; c.eps_party0 = eps_party_of(pl, party);
    set_quantiser(c, pl, party);
    const bool multik = c.K > 1;
    // the decode-side transforms carry every value divided by two (see fo_contig.h); D = (lambda / K) D_eps H^T q
    out_coef *= 2.f / (float)c.K;
    if (pl->npass == 0) {
        c.dst = out; c.len_out = len_out; c.store_mode = store_mode; c.out_coef = out_coef; c.delta = delta;
        if (multik) FO_TRY(launch(pl, KID_DEC_SINGLE, (k_contig<IN_BITS, OUT_F32, false, false, 0, true>), grid, block, st, c, none));
        else if (c.S == 10) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<10>, grid, block, st, c));
        else if (c.S == 12) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<12>, grid, block, st, c));
        else if (c.S == 14) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<14>, grid, block, st, c));
        else FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<0>, grid, block, st, c));
        return FO_OK;
    }
    if (pl->logb == 16 && !multik) {
        // blocks of exactly two tiles: one pass, a workgroup of 1024 threads per block
        c.dst = out; c.len_out = len_out; c.store_mode = store_mode; c.out_coef = out_coef; c.delta = delta;
        return launch(pl, KID_DEC_PAIR, k_decode_pair, dim3((unsigned)(pl->ntiles / 2), 1), dim3(2 * kThreads), st, c);
    }
    c.dst = tmp; c.dst_stride = 0;
    StridedArgs s = strided_base(pl, r, pl->npass - 1);
    s.dst = out; s.len_out = len_out; s.store_mode = store_mode; s.out_coef = out_coef; s.delta = delta;
    s.scales = scales; s.scales_stride = 0; s.eps_party0 = eps_party_of(pl, party);
    if (pl->npass == 1 && !multik) {
        // int16 intermediate between the two passes (padded rows when it is the plan's own buffer)
        c.dst_pad = s.src_pad = tmp == pl->buf_a ? pl->pad16 : 0u;
        FO_TRY(launch_declow(pl, grid, st, c));
        s.src = tmp;
        FO_TRY((launch_strided<SM_DEC_LAST, true>(pl, KID_DEC_HIGH, grid, st, s, none)));
        return FO_OK;
    }
    if (multik) FO_TRY(launch(pl, KID_DEC_LOW, (k_contig<IN_BITS, OUT_I32, false, false, 15, true>), grid, block, st, c, none));
    else FO_TRY(launch(pl, KID_DEC_LOW, (k_contig<IN_BITS, OUT_I32, false, false, 15>), grid, block, st, c, none));
    if (pl->npass == 1) {
        s.src = tmp;
        FO_TRY(launch_strided<SM_DEC_LAST>(pl, KID_DEC_HIGH, grid, st, s, none));
        return FO_OK;
    }
    StridedArgs s1 = strided_base(pl, r, 0);
    s1.src = tmp; s1.dst = pl->buf_c;
    FO_TRY(launch_strided<SM_MID_I32>(pl, KID_DEC_MID, grid, st, s1, none));
    s.src = pl->buf_c;
    FO_TRY(launch_strided<SM_DEC_LAST>(pl, KID_DEC_HIGH, grid, st, s, none));
    return FO_OK;
}


} // namespace fo_host
