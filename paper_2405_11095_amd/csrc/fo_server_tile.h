// Server step for transforms that fit one tile (transform length b <= 2^15, whole or blocked), in one kernel:
// for every tile, decode the M workers' messages one after the other (Def. 3.8), accumulate
// gbar = (1/M) sum_n lambda_n D_eps_n H^T q_n (eq. "server average") in registers, and re-encode the tile with
// (eps^s, lambda^s, K) (Sec. 4, "Server-to-workers encoding").  Per tile the kernel reads M * 4 KiB of packed
// signs and writes 4 KiB per bit plane; the M decoded vectors never exist in memory.
//
// The decode half is declow_tile (popcount + packed int16) with the accumulation done in its output layout; the
// encode half is the generic tile pipeline, which wants its input in its own load layout, so the mean of the
// tile makes one trip through global memory inside the kernel (128 KiB that the same workgroup reads straight
// back: a cache hit; it is also the optional gbar output).
#pragma once
#include "fo_declow.h"

namespace fo {

struct ServerTileArgs {
    ContigArgs enc;           // the re-encode: src = mean buffer (fp32 [ntot]), dst = downlink planes, scales = lambda^s
    const uint64_t *bits_up;  // [M][W]
    const float *scales_up;   // [M][nblocks]
    uint32_t M;
    float coef;               // value = lambda_n * coef * (half-valued integer): 2 / (sqrt(b) M)
};

template <bool DITHER, bool SMALLB, bool MULTIK>
__global__ __launch_bounds__(kThreads, 2) void k_server_tile(const ServerTileArgs sa, const PtrTab tab)
{
    __shared__ uint32_t lds[kLdsWords];
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const lam = reinterpret_cast<float *>(lds + kXWords + kEpsWords);
    const ContigArgs &a = sa.enc;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x;
    const uint32_t S = a.S;
    const uint64_t base = (uint64_t)tile << kTileLog2;
    const uint32_t nblk_tile = kTile >> S;
    const uint64_t blk0 = (uint64_t)tile * nblk_tile;
    const uint32_t dt = lane | (wave << 8);      // thread part of the dword index in layout LC
    const uint32_t eshift = (lane & 15u) << 1;   // bit of the pair's first coordinate inside its eps word

    float acc[64];
#pragma unroll
    for (int r = 0; r < 64; ++r) acc[r] = 0.f;

    for (uint32_t m = 0; m < sa.M; ++m) {
        // tables of worker m for this tile: 1024 eps words (256 generator calls) and one coefficient per block;
        // the barriers inside declow_tile publish them, its last one lets the next worker overwrite them
        if (t < 256u) {
            const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, m };
            uint32_t w[4];
            philox((uint32_t)(base >> 7) + t, key_eps, w);
#pragma unroll
            for (int j = 0; j < 4; ++j) epsw[t * 4u + j] = w[j];
        }
        if (t < nblk_tile) {
            const uint64_t gb = blk0 + t;
            lam[t] = gb < a.nblocks ? sa.scales_up[(uint64_t)m * a.nblocks + gb] * sa.coef : 0.f;
        }
        s16x2 v[32];
        declow_tile<0>(reinterpret_cast<const uint32_t *>(sa.bits_up + (uint64_t)m * a.W), a.W, tile, S, xbuf, v);
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            const uint32_t D = dt + declow_reg_dword(r);
            const uint32_t w = epsw[D >> 4];
            const uint32_t cbits = __float_as_uint(lam[D >> (S - 1u)]); // non-negative: the eps sign goes into bit 31
            acc[2 * r] = fmaf((float)v[r].x, __uint_as_float(((w >> eshift) << 31) | cbits), acc[2 * r]);
            acc[2 * r + 1] = fmaf((float)v[r].y, __uint_as_float(((w >> (eshift + 1u)) << 31) | cbits), acc[2 * r + 1]);
        }
        __syncthreads(); // tables read; the next worker may refill them
    }

    // the mean of the tile, natural order
    {
        float2 *gq = reinterpret_cast<float2 *>(const_cast<void *>(a.src)) + (base >> 1);
        const uint64_t room = a.len_in > base ? (a.len_in - base) >> 1 : 0; // pairs of this tile inside the buffer
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            const uint32_t D = dt + declow_reg_dword(r);
            if (D < room) gq[D] = make_float2(acc[2 * r], acc[2 * r + 1]);
        }
    }
    __syncthreads(); // workgroup-scope release / acquire: the tile is read back below by other waves

    contig_tile<IN_GRAD, OUT_PACK, DITHER, SMALLB, 0, MULTIK>(a, tab, tile, 0u, lds);
}

// Decoder of one party for transforms that fit a tile (Def. 3.8): out = lambda D_eps H^T q, first len_out
// coordinates, stored / accumulated / applied as x -= delta * value (eq. "workers update").  Uses of the
// argument block: src (packed signs), W, S, nblocks, scales (+ stride), eps_party0, the generator key,
// dst, len_out, store_mode, out_coef (for half-valued integers), delta.
__global__ __launch_bounds__(kThreads, 4) void k_decode_tile(const ContigArgs a)
{
    __shared__ uint32_t lds[kXWords + kEpsWords + kLamWords];
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const lam = reinterpret_cast<float *>(lds + kXWords + kEpsWords);
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x, slot = blockIdx.y;
    const uint32_t S = a.S;
    const uint64_t base = (uint64_t)tile << kTileLog2;
    const uint32_t nblk_tile = kTile >> S;
    const uint32_t dt = lane | (wave << 8);
    const uint32_t eshift = (lane & 15u) << 1;
    const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;

    if (t < 256u) {
        const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, eps_party };
        uint32_t w[4];
        philox((uint32_t)(base >> 7) + t, key_eps, w);
#pragma unroll
        for (int j = 0; j < 4; ++j) epsw[t * 4u + j] = w[j];
    }
    if (t < nblk_tile) {
        const uint64_t gb = (uint64_t)tile * nblk_tile + t;
        lam[t] = gb < a.nblocks ? a.scales[slot * a.scales_stride + gb] * a.out_coef : 0.f;
    }
    s16x2 v[32];
    const uint32_t *words = reinterpret_cast<const uint32_t *>(static_cast<const uint64_t *>(a.src) + slot * a.src_stride);
    declow_tile<0>(words, a.W, tile, S, xbuf, v); // its barriers publish the tables

    float2 *dst = reinterpret_cast<float2 *>(static_cast<float *>(a.dst) + base);
    const uint64_t room = a.len_out > base ? a.len_out - base : 0; // valid coordinates of this tile
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const uint32_t D = dt + declow_reg_dword(r);
        const uint32_t w = epsw[D >> 4];
        const uint32_t cbits = __float_as_uint(lam[D >> (S - 1u)]);
        const float y0 = (float)v[r].x * __uint_as_float(((w >> eshift) << 31) | cbits);
        const float y1 = (float)v[r].y * __uint_as_float(((w >> (eshift + 1u)) << 31) | cbits);
        if (2ull * D + 1 < room) {
            float2 q = dst[D];
            if (a.store_mode == STORE_SET) q = make_float2(y0, y1);
            else if (a.store_mode == STORE_ACC) q = make_float2(q.x + y0, q.y + y1);
            else q = make_float2(q.x - a.delta * y0, q.y - a.delta * y1);
            dst[D] = q;
        } else if (2ull * D < room) {
            float &q = static_cast<float *>(a.dst)[base + 2ull * D];
            if (a.store_mode == STORE_SET) q = y0;
            else if (a.store_mode == STORE_ACC) q += y0;
            else q -= a.delta * y0;
        }
    }
}

} // namespace fo
