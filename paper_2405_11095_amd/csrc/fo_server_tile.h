// Kernels for transforms that fit one tile (transform length b <= 2^15, whole or blocked), built on declow_tile
// (popcount + packed int16) with the amplitude, the eps flip and the store or accumulation done in its output
// layout.
//   k_mean_tile  : the server's mean gbar = (1/M) sum_n lambda_n D_eps_n H^T q_n (Def. 3.8, eq. "server average"):
//                  per tile, the M messages are decoded one after the other and summed in registers; the M decoded
//                  vectors never exist in memory (M * 4 KiB of packed signs in, 128 KiB of fp32 out per tile).
//                  The re-encode of the mean is the ordinary encode kernel.  (A variant that also re-encoded the
//                  tile in the same kernel was measured slower: it needs so many registers that one 512-thread
//                  workgroup fills a CU.)
//   k_decode_tile: one party's decoder with store / accumulate / SGD update.
//   k_decode_pair: the decoder for transforms of exactly 2^16 points: a workgroup of 1024 threads, two groups of
//                  512 on the two tiles of a block, sixteenth stage through both groups' exchange buffers
//                  (declow_pair_back).  One pass over the packed signs instead of an int16 intermediate and a
//                  strided second pass.  (The same construction for the server's mean was measured no faster
//                  than the two-pass path, whose second pass also starts the re-encode.)
#pragma once
#include "fo_declow.h"

namespace fo {

struct ServerTileArgs {
    ContigArgs enc;           // geometry and generator key; src = mean buffer (fp32 [len_in], written here)
    const uint64_t *bits_up;  // [M][W]
    const float *scales_up;   // [M][nblocks]
    uint32_t M;
    float coef;               // value = lambda_n * coef * (half-valued integer): 2 / (sqrt(b) M)
};

// SC: compiled for transforms of 2^SC points (the block lengths of the blocked workload), 0: length read at run time.
template <int SC>
__global__ __launch_bounds__(kThreads, 4) void k_mean_tile(const ServerTileArgs sa)
{
    // two sets of tables used in turn, so that the worker loop needs no barrier of its own
    __shared__ uint32_t lds[kXWords + 2 * (kEpsWords + kLamWords)];
    uint32_t *const xbuf = lds;
    uint32_t *const tables = lds + kXWords;
    const ContigArgs &a = sa.enc;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x;
    const uint32_t S = SC ? (uint32_t)SC : a.S;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    const uint64_t base = (uint64_t)tile << kTileLog2;
    const uint32_t nblk_tile = kTile >> S;
    const uint64_t blk0 = (uint64_t)tile * nblk_tile;
    const uint32_t dt = lane | (wave << 8);      // thread part of the dword index in layout LC
    const uint32_t eshift = (lane & 15u) << 1;   // bit of the pair's first coordinate inside its eps word

    float acc[64];
#pragma unroll
    for (int r = 0; r < 64; ++r) acc[r] = 0.f;

    for (uint32_t m = 0; m < sa.M; ++m) {
        // tables of worker m for this tile: 1024 eps words (256 generator calls) and one coefficient per block.
        // The barriers inside declow_tile publish them; every wave passes those only when it is done with worker
        // m-1, so the set of worker m-2 may be overwritten without waiting.
        uint32_t *const epsw = tables + (m & 1u) * (kEpsWords + kLamWords);
        float *const lam = reinterpret_cast<float *>(epsw + kEpsWords);
        if (t < 256u) {
            const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, m };
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
        uint32_t tl = t;
        asm volatile("" : "+v"(tl));
        declow_tile<SC>(reinterpret_cast<const uint32_t *>(sa.bits_up + (uint64_t)m * a.W), a.W, tile, S, xbuf, xbuf, v, tl);
        __syncthreads(); // the exchange buffer is read; the next worker's first exchange may write it
        // the table addresses are recomputed for every worker: hoisted out of the loop they would hold 64 registers
        // next to the 64 accumulators
        uint32_t dtl = dt;
        asm volatile("" : "+v"(dtl));
#pragma unroll
        for (int r = 0; r < 32; ++r) {
            const uint32_t D = dtl + declow_reg_dword(r);
            const uint32_t w = epsw[D >> 4];
            const uint32_t cbits = __float_as_uint(lam[D >> (S - 1u)]); // the eps bit is added into bit 31: a flip of the sign, whatever it was
            acc[2 * r] = fmaf((float)v[r].x, __uint_as_float(((w >> eshift) << 31) + cbits), acc[2 * r]);
            acc[2 * r + 1] = fmaf((float)v[r].y, __uint_as_float(((w >> (eshift + 1u)) << 31) + cbits), acc[2 * r + 1]);
        }
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
}

// Decoder of one party for transforms that fit a tile (Def. 3.8): out = lambda D_eps H^T q, first len_out
// coordinates, stored / accumulated / applied as x -= delta * value (eq. "workers update").  Uses of the
// argument block: src (packed signs), W, S, nblocks, scales (+ stride), eps_party0, the generator key,
// dst, len_out, store_mode, out_coef (for half-valued integers), delta.
template <int SC>
__global__ __launch_bounds__(kThreads, 4) void k_decode_tile(const ContigArgs a)
{
    __shared__ uint32_t lds[kXWords + kEpsWords + kLamWords];
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const lam = reinterpret_cast<float *>(lds + kXWords + kEpsWords);
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x, slot = blockIdx.y;
    const uint32_t S = SC ? (uint32_t)SC : a.S;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    const uint64_t base = (uint64_t)tile << kTileLog2;
    const uint32_t nblk_tile = kTile >> S;
    const uint32_t dt = lane | (wave << 8);
    const uint32_t eshift = (lane & 15u) << 1;
    const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;

    if (t < 256u) {
        const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, eps_party };
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
    declow_tile<SC>(words, a.W, tile, S, xbuf, xbuf, v); // its barriers publish the tables

    float2 *dst = reinterpret_cast<float2 *>(static_cast<float *>(a.dst) + base);
    const uint64_t room = a.len_out > base ? a.len_out - base : 0; // valid coordinates of this tile
#pragma unroll
    for (int r = 0; r < 32; ++r) {
        const uint32_t D = dt + declow_reg_dword(r);
        const uint32_t w = epsw[D >> 4];
        const uint32_t cbits = __float_as_uint(lam[D >> (S - 1u)]);
        const float y0 = (float)v[r].x * __uint_as_float(((w >> eshift) << 31) + cbits);
        const float y1 = (float)v[r].y * __uint_as_float(((w >> (eshift + 1u)) << 31) + cbits);
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

// Geometry of one group of a pair workgroup.
struct PairGroup {
    uint32_t h, t, lane, wave, tile;
    uint64_t base;
    uint32_t dt, eshift;
};
__device__ __forceinline__ PairGroup pair_group()
{
    PairGroup g;
    g.h = __builtin_amdgcn_readfirstlane(threadIdx.x >> 9); // the same in every lane of a wave: branches on it are scalar
    g.t = threadIdx.x & 511u;
    g.lane = g.t & 63u;
    g.wave = g.t >> 6;
    g.tile = 2u * blockIdx.x + g.h;
    g.base = (uint64_t)g.tile << kTileLog2;
    g.dt = g.lane | (g.wave << 8);
    g.eshift = (g.lane & 15u) << 1;
    return g;
}

// k_decode_tile for transforms of exactly 2^16 points; same uses of the argument block.
static __global__ __launch_bounds__(2 * kThreads) void k_decode_pair(const ContigArgs a)
{
    __shared__ uint32_t lds[2 * (kXWords + kEpsWords)];
    const PairGroup g = pair_group();
    const uint32_t slot = blockIdx.y;
    uint32_t *const xb_own = lds + g.h * kXWords;
    const uint32_t *const xb_oth = lds + (g.h ^ 1u) * kXWords;
    uint32_t *const epsw = lds + 2 * kXWords + g.h * kEpsWords;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;
    const uint64_t gb = g.base >> 16;

    if (g.t < 256u) {
        const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, eps_party };
        uint32_t w[4];
        philox((uint32_t)(g.base >> 7) + g.t, key_eps, w);
#pragma unroll
        for (int j = 0; j < 4; ++j) epsw[g.t * 4u + j] = w[j];
    }
    const float lamc = gb < a.nblocks ? a.scales[slot * a.scales_stride + gb] * a.out_coef : 0.f;
    const uint32_t cbits = __float_as_uint(lamc);
    {
        s16x2 v[32];
        const uint32_t *words = reinterpret_cast<const uint32_t *>(static_cast<const uint64_t *>(a.src) + slot * a.src_stride);
        declow_front<15>(words, a.W, g.tile, 15u, xb_own, xb_own, v, g.t); // its barriers publish the eps table
    }
    float2 *dst = reinterpret_cast<float2 *>(static_cast<float *>(a.dst) + g.base);
    const uint64_t room = a.len_out > g.base ? a.len_out - g.base : 0; // valid coordinates of this tile
    auto store = [&](auto G, const int32_t (&w)[16]) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t D = g.dt + declow_reg_dword(8 * decltype(G)::value + q);
            const uint32_t e = epsw[D >> 4];
            const float y0 = (float)w[2 * q] * __uint_as_float(((e >> g.eshift) << 31) + cbits);
            const float y1 = (float)w[2 * q + 1] * __uint_as_float(((e >> (g.eshift + 1u)) << 31) + cbits);
            if (2ull * D + 1 < room) {
                float2 o = dst[D];
                if (a.store_mode == STORE_SET) o = make_float2(y0, y1);
                else if (a.store_mode == STORE_ACC) o = make_float2(o.x + y0, o.y + y1);
                else o = make_float2(o.x - a.delta * y0, o.y - a.delta * y1);
                dst[D] = o;
            } else if (2ull * D < room) {
                float &o = static_cast<float *>(a.dst)[g.base + 2ull * D];
                if (a.store_mode == STORE_SET) o = y0;
                else if (a.store_mode == STORE_ACC) o += y0;
                else o -= a.delta * y0;
            }
        }
    };
    if (g.h) declow_pair_back<true>(xb_own, xb_oth, g.t, store);
    else declow_pair_back<false>(xb_own, xb_oth, g.t, store);
}

} // namespace fo
