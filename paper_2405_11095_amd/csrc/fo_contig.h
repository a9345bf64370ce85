// Contiguous-tile kernel: the low min(log2 b, 15) Walsh-Hadamard stages of every 2^15-coordinate
// tile, fused with whatever sits at either end of the transform:
//   input  : fp32 gradient (zero-padded) with the eps sign flip and the per-block sum of squares
//            (Def. 3.5; norm for the amplitude of Thm 5.5) | fp32 intermediate | packed sign bits |
//            the M workers' packed sign bits summed per coordinate (vertical popcount; valid when all
//            workers share one eps and one amplitude, because H^T is linear: sum_n H^T q_n = H^T sum_n q_n)
//   output : dither + sign + 64-bit packing (Def. 3.2, Def. 3.7) | int32 intermediate |
//            amplitude scaling + eps flip + store / accumulate / SGD update (Def. 3.8, Sec. 4)
//
// Index-bit choreography for a tile (b0..b14 = bits of the tile-local coordinate):
//   L0 (global loads, 16 B per lane): regs = (b0,b1,b8,b9,b10,b11) lanes = (b2..b7)   waves = (b12,b13,b14)
//   L1 (after the intra-wave exchange): regs = (b2..b7)            lanes = (b0,b1,b8,b9,b10,b11)
//   L2 (after the cross-wave exchange): regs = (b6,b8,b12,b13,b14,b7) lanes = (b0..b5) waves = (b9,b10,b11)
// (OUT_I16 reads the second exchange as lanes = (b1..b6), regs = (b0,b8,b12,b13,b14,b7) instead, so that a
// thread owns pairs of neighbouring coordinates and stores them as one dword.)
// The decode side (IN_BITS) carries every value divided by two: the stage on b0 is fused into the
// unpacking as (c0 + c1 - 1, c0 - c1) for sign bits c0, c1, which is half the butterfly of the +-1
// values, so after all fifteen stages the values fit int16 exactly; consumers fold the factor two
// into their scale.
// In L2 a wave holds 64 consecutive coordinates per register, so one compare per register yields
// a packed 64-bit word, and the four registers that differ in (b6,b7) share one dither draw.
// b7 keeps register bit 5 across the second exchange, so each half of it can run in place.
#pragma once
#include "fo_device.h"

namespace fo {

enum { IN_GRAD = 0, IN_F32 = 1, IN_BITS = 2, IN_COUNT = 3 };
enum { OUT_PACK = 0, OUT_I32 = 1, OUT_F32 = 2, OUT_I16 = 3 };
enum { STORE_SET = 0, STORE_ACC = 1, STORE_AXPY = 2 };

struct PtrTab {
    const float *p[64];
};

struct ContigArgs {
    const void *src;        // IN_F32: fp32 [slot][ntot]; IN_BITS: uint64 [slot][W]; IN_GRAD: unused if use_tab
    uint64_t src_stride;    // elements between party slots
    void *dst;              // OUT_PACK: uint64 [slot][W]; OUT_I32 / OUT_I16: int [slot][ntot]; OUT_F32: fp32 [len_out]
    uint64_t dst_stride;
    float *scales;          // [slot][nblocks]
    uint64_t scales_stride;
    uint64_t len_in;        // valid input coordinates (IN_GRAD)
    uint64_t len_out;       // valid output coordinates (OUT_F32)
    uint64_t W;             // packed words per party
    uint64_t nblocks;
    uint32_t S;             // stages inside the tile = min(log2 b, 15)
    uint32_t logb;          // log2 of the transform length
    uint32_t use_tab;       // IN_GRAD: take the source pointer of slot y from the pointer table
    uint32_t compute_scale; // IN_GRAD: derive lambda from the measured block norm (else read scales[])
    uint32_t dither;        // 0 uniform, 1 none
    uint32_t store_mode;    // OUT_F32: STORE_*
    uint32_t M;             // IN_COUNT: number of packed vectors to add up
    uint32_t K;             // MULTIK: averaging count of the quantiser (Def. 3.2) being applied / decoded
    uint32_t planes;        // MULTIK: bit planes of the message, ceil(log2(K + 1)); plane p starts at word p * W
    uint32_t scales_only;   // IN_GRAD: write the blocks' amplitudes and stop (no transform)
    uint32_t tile0;         // first tile of this launch (a launch may cover a range of tiles)
    uint32_t src_pad;       // IN_F32: tile t of the intermediate starts at t * (2^15 + src_pad) (see StridedArgs)
    uint32_t dst_pad;       // k_declow: the same for its int16 output
    uint32_t party0;        // party id of slot 0 (slot y is party0 + y); FO_PARTY_SERVER stays as is
    uint32_t eps_party0;    // same for the eps stream
    uint32_t k0, k1, round_lo;
    const unsigned long long *round_dev; // optional: round counter read at run time (see resolve_round)
    float coef_lambda;      // alpha * sqrt(ln b / b)
    float sqrtb;            // threshold in the unnormalised domain = lambda * sqrt(b)
    float out_coef;         // OUT_F32: value = lambda * out_coef * (H^T q)_i  (1/sqrt(b), times 1/M on the server)
    float delta;            // STORE_AXPY: x -= delta * value
    unsigned long long *stat_clipped; // OUT_PACK, optional: per slot, += #{i : |z_i| > lambda} (flattening failed there)
    unsigned long long *stat_near;    // OUT_PACK, optional: per slot, += #{i : |z_i + tau_i| < 1e-6 lambda} (first dither)
};

// DITHER: uniform dither on (OUT_PACK only).  SMALLB: transform length 64 or 128, where the four
// registers that share a dither draw belong to different blocks.  Both are compile-time so that the
// per-value code is branch free.
// SC > 0: compiled for exactly SC stages inside the tile (SC = 15: transform length >= 2^15), which
// makes every stage unconditional; SC = 0 reads the stage count from the arguments.
// STATS: OUT_PACK also adds to the caller's diagnostic counters (see fo_stats).
// MULTIK: the K-fold averaged quantiser of Def. 3.2 (the server's message when K > 1).  Coordinate i carries
// c_i = #{k < K : z_i + tau_{k,i} >= 0} in {0..K}, i.e. q_i = 2 c_i - K = (K / lambda) Q_{lambda,K}(z)_i, stored as
// `planes` bit planes of W words each (plane p holds bit p of every c_i).  OUT_PACK draws K dithers per
// coordinate and writes the planes; IN_BITS reads them.  K = 1 is the plain sign message and uses MULTIK = false.
// The work of 512 threads (t = 0..511) on tile `tile` of party slot `slot`; lds has kLdsWords words.
// PAIR (gradient in, transform length exactly 2^16): two such groups of 512 threads in one workgroup take the two
// tiles of a block; lds_partner is the other group's LDS.  The stage on bit 15 pairs coordinate i of the lower
// tile with coordinate i of the upper one, and it can go first: each group loads and flips its own tile, the two
// swap their values through LDS, the lower forms x_lo + x_hi and the upper x_lo - x_hi, and each runs the fifteen
// remaining stages on its own tile as usual.  The 2^16-point transform then costs one pass over memory instead
// of two.  The block's norm is the sum of the two groups' partial sums.
template <int IN, int OUT, bool DITHER, bool SMALLB, int SC, bool MULTIK, bool STATS = false, bool PAIR = false, bool GUARDED = true>
__device__ __forceinline__ void contig_tile(const ContigArgs &a, const PtrTab &tab, const uint32_t tile, const uint32_t slot,
                                            uint32_t *const lds, const uint32_t t, uint32_t *const lds_partner = nullptr)
{
    static_assert(!PAIR || (IN == IN_GRAD && OUT == OUT_PACK && SC == 15 && !SMALLB), "pair mode: gradient in, bits out");
    using T = typename std::conditional<(IN == IN_BITS || IN == IN_COUNT), int32_t, float>::type;
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const lam = reinterpret_cast<float *>(lds + kXWords + kEpsWords);
    float *const red = reinterpret_cast<float *>(lds + kXWords + kEpsWords + kLamWords);
    // PAIR: the partial sums of the block's lower and upper tile, so that both groups add them in the same order
    const float *const red_lo = PAIR ? reinterpret_cast<const float *>(((tile & 1u) ? lds_partner : lds) + kXWords + kEpsWords + kLamWords) : nullptr;
    const float *const red_hi = PAIR ? reinterpret_cast<const float *>(((tile & 1u) ? lds : lds_partner) + kXWords + kEpsWords + kLamWords) : nullptr;

    const uint32_t lane = t & 63u, wave = t >> 6;
    const uint64_t base = (uint64_t)tile << kTileLog2;
    const uint32_t S = SC ? (uint32_t)SC : a.S;
    const uint32_t party = (a.party0 == 0xFFFFFFFFu) ? a.party0 : a.party0 + slot;
    const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, eps_party };
    const RngKey key_dit = { a.k0, rk1, kDomainDither, rlo, party };

    T v[kV];

    // ------------------------------------------------------------------ input, layout L0
    if constexpr (IN == IN_GRAD || IN == IN_F32) {
        const float *src = (IN == IN_GRAD && a.use_tab) ? tab.p[slot]
                                                        : static_cast<const float *>(a.src) + slot * a.src_stride;
        // GUARDED = false: the caller vouches that the whole tile lies inside the input (no per-chunk checks)
        const uint64_t limit = (IN == IN_GRAD && GUARDED) ? a.len_in : ~0ull;
        if constexpr (IN == IN_F32) src += (uint64_t)tile * a.src_pad;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const uint64_t i = base + wave * 4096u + c * 256u + lane * 4u;
            float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i + 3 < limit) {
                x = *reinterpret_cast<const float4 *>(src + i);
            } else {
                if (i < limit) x.x = src[i];
                if (i + 1 < limit) x.y = src[i + 1];
                if (i + 2 < limit) x.z = src[i + 2];
            }
            v[4 * c + 0] = x.x; v[4 * c + 1] = x.y; v[4 * c + 2] = x.z; v[4 * c + 3] = x.w;
        }
    } else if constexpr (IN == IN_COUNT) {
        // q_sum_i = sum_n q_{n,i} = 2 * popcount_i - M.  The four coordinates of a lane are a nibble of one
        // 32-bit half word; multiplying the nibble by 0x00204081 puts its bits into the low bit of four
        // bytes, so one add per worker counts four coordinates at once (M <= 64 < 256: no byte overflows).
        const uint32_t *src = static_cast<const uint32_t *>(a.src);
        uint32_t cnt[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) cnt[c] = 0u;
        for (uint32_t m = 0; m < a.M; ++m) {
            const uint32_t *sm = src + 2 * (uint64_t)m * a.src_stride;
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                const uint64_t gh = 2 * ((uint64_t)tile * 512u + wave * 64u + c * 4u) + (lane >> 3); // 32-bit half word
                const uint32_t h = (gh < 2 * a.W) ? sm[gh] : 0u;
                cnt[c] += (((h >> ((lane & 7u) * 4u)) & 15u) * 0x00204081u) & 0x01010101u;
            }
        }
#pragma unroll
        for (int c = 0; c < 16; ++c)
#pragma unroll
            for (int k = 0; k < 4; ++k) v[4 * c + k] = 2 * (int32_t)((cnt[c] >> (8 * k)) & 255u) - (int32_t)a.M;
    } else {
        const uint64_t *src = static_cast<const uint64_t *>(a.src) + slot * a.src_stride;
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const uint64_t gw = (uint64_t)tile * 512u + wave * 64u + c * 4u + (lane >> 4);
            // half of the b0 butterfly of the values 2 c - K: sum / 2 = c0 + c1 - K, difference / 2 = c0 - c1
            int32_t c0, c1, c2, c3, K = 1;
            if constexpr (MULTIK) {
                c0 = c1 = c2 = c3 = 0;
                K = (int32_t)a.K;
                for (uint32_t p = 0; p < a.planes; ++p) {
                    const uint64_t w = (gw < a.W) ? src[p * a.W + gw] : 0ull;
                    const uint32_t nib = (uint32_t)(w >> ((lane & 15u) * 4u));
                    c0 += (int32_t)((nib & 1u) << p);
                    c1 += (int32_t)(((nib >> 1) & 1u) << p);
                    c2 += (int32_t)(((nib >> 2) & 1u) << p);
                    c3 += (int32_t)(((nib >> 3) & 1u) << p);
                }
            } else {
                const uint64_t w = (gw < a.W) ? src[gw] : 0ull;
                const uint32_t nib = (uint32_t)(w >> ((lane & 15u) * 4u));
                c0 = nib & 1u, c1 = (nib >> 1) & 1u, c2 = (nib >> 2) & 1u, c3 = (nib >> 3) & 1u;
            }
            v[4 * c + 0] = c0 + c1 - K;
            v[4 * c + 1] = c0 - c1;
            v[4 * c + 2] = c2 + c3 - K;
            v[4 * c + 3] = c2 - c3;
        }
    }

    if constexpr (IN == IN_GRAD) {
        // per-block sum of squares of the raw gradient (sign flips do not change it)
        if (a.compute_scale) {
            const uint32_t G = S < 12u ? S : 12u;        // segment = 2^G coordinates, inside one wave and one block
            const uint32_t segs_per_wave = 4096u >> G;
            float acc = 0.f;
            if (S >= 8u) {
                const uint32_t cps = 1u << (G - 8u);      // chunks per segment
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    acc += (v[4 * c] * v[4 * c] + v[4 * c + 1] * v[4 * c + 1]) +
                           (v[4 * c + 2] * v[4 * c + 2] + v[4 * c + 3] * v[4 * c + 3]);
                    if (((c + 1) & (cps - 1u)) == 0u) {
                        const float s = wave_sum(acc, 6);
                        if (lane == 0) red[wave * segs_per_wave + ((uint32_t)c >> (G - 8u))] = s;
                        acc = 0.f;
                    }
                }
            } else {
                const uint32_t lanes_log2 = S - 2u;       // lanes per segment: 16 or 32
#pragma unroll
                for (int c = 0; c < 16; ++c) {
                    const float p = (v[4 * c] * v[4 * c] + v[4 * c + 1] * v[4 * c + 1]) +
                                    (v[4 * c + 2] * v[4 * c + 2] + v[4 * c + 3] * v[4 * c + 3]);
                    const float s = wave_sum(p, (int)lanes_log2);
                    if ((lane & ((1u << lanes_log2) - 1u)) == 0u)
                        red[wave * segs_per_wave + c * (256u >> S) + (lane >> lanes_log2)] = s;
                }
            }
        }
        if (a.scales_only) {
            // amplitudes only (used to agree on a common amplitude before any worker quantises)
            __syncthreads();
            if constexpr (PAIR) {
                if (t == 0 && !(tile & 1u)) {
                    float s = 0.f;
                    for (uint32_t k = 0; k < 8u; ++k) s += red_lo[k];
                    for (uint32_t k = 0; k < 8u; ++k) s += red_hi[k];
                    const uint64_t gb = base >> 16;
                    if (gb < a.nblocks) a.scales[slot * a.scales_stride + gb] = a.coef_lambda * sqrtf(s);
                }
                return;
            }
            const uint32_t nblk = kTile >> S;
            if (t < nblk) {
                const uint64_t gb = (uint64_t)tile * nblk + t;
                float s;
                if (S <= 12u) {
                    s = red[t];
                } else {
                    const uint32_t per = 1u << (S - 12u);
                    s = 0.f;
                    for (uint32_t k = 0; k < per; ++k) s += red[t * per + k];
                }
                if (gb < a.nblocks) a.scales[slot * a.scales_stride + gb] = a.coef_lambda * sqrtf(s);
            }
            return;
        }
        // eps flip: lanes 0..31 of each wave draw the 32 generator blocks covering the wave's 4096 coordinates
        if (lane < 32u) {
            uint32_t w[4];
            philox((uint32_t)((base + wave * 4096u) >> 7) + lane, key_eps, w);
#pragma unroll
            for (int j = 0; j < 4; ++j) epsw[wave * 128u + lane * 4u + j] = w[j];
        }
        wave_sync();
#pragma unroll
        for (int c = 0; c < 16; ++c) {
            const uint32_t nib = epsw[wave * 128u + c * 8u + (lane >> 3)] >> ((lane & 7u) * 4u);
#pragma unroll
            for (int k = 0; k < 4; ++k) v[4 * c + k] = flip_by_bit31(v[4 * c + k], nib << (31 - k));
        }
        if constexpr (PAIR) {
            // stage b15 across the two groups, sixteen values per thread and round.  Two buffers in turn: the
            // barrier of round g+1 comes after every thread's reads of round g, so round g+2 may overwrite them.
            const uint32_t upper = tile & 1u;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float4 *const mine = reinterpret_cast<float4 *>(xbuf + (g & 1) * 8192u) + t;
                const float4 *const theirs = reinterpret_cast<const float4 *>(lds_partner + (g & 1) * 8192u) + t;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    mine[c * 512] = make_float4(v[16 * g + 4 * c], v[16 * g + 4 * c + 1], v[16 * g + 4 * c + 2], v[16 * g + 4 * c + 3]);
                __syncthreads();
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const float4 o = theirs[c * 512];
                    const float ov[4] = { o.x, o.y, o.z, o.w };
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        float &x = v[16 * g + 4 * c + k];
                        x = upper ? ov[k] - x : x + ov[k];
                    }
                }
            }
            __syncthreads(); // the last reads are done before the first exchange of the transform writes xbuf
        }
    }

    // ------------------------------------------------------------------ first register round: b0,b1,b8..b11
    if constexpr (IN != IN_BITS) bfly<T, 0>(v); // the decode side did this stage while unpacking
    bfly<T, 1>(v);
    if (S > 8u) bfly<T, 2>(v);
    if (S > 9u) bfly<T, 3>(v);
    if (S > 10u) bfly<T, 4>(v);
    if (S > 11u) bfly<T, 5>(v);

    // ------------------------------------------------------------------ exchange L0 -> L1 (inside each wave)
    {
        uint32_t *const wb = xbuf + wave * 2112u + (lane >> 5) * 1056u;
        const uint32_t col = lane & 31u;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
            for (int r = 0; r < 32; ++r) wb[r * 33 + col] = __builtin_bit_cast(uint32_t, v[sub * 32 + r]);
            wave_sync();
#pragma unroll
            for (int r = 0; r < 32; ++r) v[sub * 32 + r] = __builtin_bit_cast(T, wb[col * 33 + r]);
            wave_sync();
        }
        swap_reg5_lane5(v);
    }

    // ------------------------------------------------------------------ second register round: b2..b7
    bfly<T, 0>(v);
    bfly<T, 1>(v);
    bfly<T, 2>(v);
    bfly<T, 3>(v);
    if (S > 6u) bfly<T, 4>(v);
    if (S > 7u) bfly<T, 5>(v);

    __syncthreads();

    // ------------------------------------------------------------------ amplitudes of the tile's blocks
    const uint32_t nblk_tile = kTile >> S;
    const uint64_t blk0 = (a.logb <= (uint32_t)kTileLog2) ? (uint64_t)tile * nblk_tile : (base >> a.logb);
    if constexpr (OUT == OUT_PACK || OUT == OUT_F32) { // the integer intermediates carry no amplitude
        if (t < nblk_tile) {
            float l = 0.f;
            const uint64_t gb = blk0 + t;
            if (IN == IN_GRAD && a.compute_scale) {
                float s;
                if constexpr (PAIR) {
                    s = 0.f;
                    for (uint32_t k = 0; k < 8u; ++k) s += red_lo[k];
                    for (uint32_t k = 0; k < 8u; ++k) s += red_hi[k];
                } else if (S <= 12u) {
                    s = red[t];
                } else {
                    const uint32_t per = 1u << (S - 12u);
                    s = 0.f;
                    for (uint32_t k = 0; k < per; ++k) s += red[t * per + k];
                }
                l = a.coef_lambda * sqrtf(s);
                if (gb < a.nblocks && !(PAIR && (tile & 1u))) a.scales[slot * a.scales_stride + gb] = l;
            } else if (gb < a.nblocks) {
                l = a.scales[slot * a.scales_stride + gb];
            }
            // the plain sign quantiser compares in the integer domain and wants -128 / (lambda sqrt(b) 2^-24) (see below)
            if constexpr (OUT == OUT_PACK && DITHER && !MULTIK && !STATS) l = -128.f / (l * (a.sqrtb * 5.9604644775390625e-08f));
            lam[t] = l;
        }
    }
    if constexpr (OUT == OUT_F32) {
        // eps words for layout L2: lane q < 32 of wave w draws the generator block that covers
        // (b8,b12,b13,b14) = q & 15, b7 = q >> 4, (b9..b11) = w
        if (lane < 32u) {
            uint32_t w[4];
            const uint32_t call = (lane >> 4) | ((lane & 1u) << 1) | (wave << 2) | (((lane >> 1) & 7u) << 5);
            philox((uint32_t)(base >> 7) + call, key_eps, w);
#pragma unroll
            for (int j = 0; j < 4; ++j) epsw[wave * 128u + lane * 4u + j] = w[j];
        }
    }

    // ------------------------------------------------------------------ exchange L1 -> L2 (whole workgroup)
    {
        const uint32_t wofs = (lane & 3u) + ((lane >> 2) | (wave << 4)) * 132u;
        const uint32_t rofs = lane + wave * 264u;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
            if (sub) __syncthreads();
#pragma unroll
            for (int r = 0; r < 32; ++r) xbuf[wofs + r * 4] = __builtin_bit_cast(uint32_t, v[sub * 32 + r]);
            __syncthreads();
            if constexpr (OUT == OUT_I16) {
                // lanes = (b1..b6): a lane reads the pair b0 = 0, 1 (8 bytes); register sub*32 + q = (b0,b8,b12,b13,b14 | b7)
                const uint2 *rp2 = reinterpret_cast<const uint2 *>(xbuf) + (lane + wave * 132u);
#pragma unroll
                for (int q = 0; q < 32; q += 2) {
                    const uint2 d = rp2[(((q >> 1) & 1) + (q >> 2) * 16) * 66];
                    v[sub * 32 + q] = __builtin_bit_cast(T, d.x);
                    v[sub * 32 + q + 1] = __builtin_bit_cast(T, d.y);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 32; ++q) // register sub*32 + q = (b6,b8,b12,b13,b14 | b7 = sub)
                    v[sub * 32 + q] =
                        __builtin_bit_cast(T, xbuf[rofs + (q & 1) * 64 + (((q >> 1) & 1) + (q >> 2) * 16) * 132]);
            }
        }
    }

    // ------------------------------------------------------------------ third register round: b12,b13,b14
    if (S > 12u) bfly<T, 2>(v);
    if (S > 13u) bfly<T, 3>(v);
    if (S > 14u) bfly<T, 4>(v);

    // tile-local coordinate of register r in L2
    auto local_of = [&](int r) -> uint32_t {
        return lane | ((uint32_t)(r & 1) << 6) | ((uint32_t)(r >> 5) << 7) | ((uint32_t)((r >> 1) & 1) << 8) | (wave << 9) |
               ((uint32_t)((r >> 2) & 7) << 12);
    };

    // ------------------------------------------------------------------ output
    if constexpr (OUT == OUT_PACK && STATS) {
        // Diagnostic counters: a second sweep over the registers, compiled only into the variants that are
        // launched while a stats block is attached (it would cost the others registers).
        if (a.stat_clipped) {
            uint32_t clipped = 0u, near = 0u;
            const float tscale = a.sqrtb * 5.9604644775390625e-08f;
#pragma unroll
            for (int g = 0; g < 16; ++g) {
                uint32_t w[4] = { 0u, 0u, 0u, 0u };
                if constexpr (DITHER) philox((uint32_t)(((base + local_of(2 * g)) >> 8) << 6) | lane, key_dit, w);
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int r = 2 * g + (s & 1) + 32 * (s >> 1);
                    const float l = lam[local_of(r) >> S];
                    float tv = v[r];
                    if constexpr (DITHER) tv = fmaf(l * tscale, fmaf((float)(w[s] >> 8), 2.f, -16777215.f), tv);
                    clipped += (uint32_t)__popcll(__ballot(fabsf(v[r]) > l * a.sqrtb));
                    near += (uint32_t)__popcll(__ballot(fabsf(tv) < 1e-6f * l * a.sqrtb));
                }
            }
            if (lane == 0u) {
                atomicAdd(a.stat_clipped + slot, (unsigned long long)clipped);
                atomicAdd(a.stat_near + slot, (unsigned long long)near);
            }
        }
    }
    if constexpr (OUT == OUT_PACK && MULTIK) {
        uint32_t lo[8], hi[8]; // lane j: word of register j, one pair per bit plane
#pragma unroll
        for (int p = 0; p < 8; ++p) lo[p] = hi[p] = 0u;
        const float tscale = a.sqrtb * 5.9604644775390625e-08f; // 2^-24: u = m * 2^-24 with m odd
        static_for<16>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            const uint32_t lg = local_of(2 * g); // b6 = b7 = 0
            float thr_g = 0.f;
            if constexpr (DITHER && !SMALLB) thr_g = lam[lg >> S] * tscale;
            uint32_t cnt[4] = { 0u, 0u, 0u, 0u };
            for (uint32_t k = 0; k < a.K; ++k) {
                uint32_t w[4] = { 0u, 0u, 0u, 0u };
                if constexpr (DITHER) {
                    const RngKey key_k = { key_dit.k0, key_dit.k1, kDomainDither | (k << 8), key_dit.c2, key_dit.c3 };
                    philox((uint32_t)(((base + lg) >> 8) << 6) | lane, key_k, w);
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    const int r = 2 * g + (s & 1) + 32 * (s >> 1); // slot s = b6 | b7 << 1
                    float tv = v[r];
                    if constexpr (DITHER) {
                        float thr = thr_g;
                        if constexpr (SMALLB) thr = lam[local_of(r) >> S] * tscale;
                        const float m = fmaf((float)(w[s] >> 8), 2.f, -16777215.f);
                        tv = fmaf(thr, m, tv);
                    }
                    cnt[s] += (tv >= 0.f) ? 1u : 0u;
                }
            }
            static_for<8>([&](auto pc) {
                constexpr int p = decltype(pc)::value;
                if ((uint32_t)p < a.planes) {
                    uint64_t word[4];
#pragma unroll
                    for (int s = 0; s < 4; ++s) word[s] = __ballot(((cnt[s] >> p) & 1u) != 0u);
                            static_for<4>([&](auto sc) {
                        constexpr int s = decltype(sc)::value;
                        constexpr int r = 2 * g + (s & 1) + 32 * (s >> 1);
                        lo[p] = write_lane<r>(lo[p], (uint32_t)word[s]);
                        hi[p] = write_lane<r>(hi[p], (uint32_t)(word[s] >> 32));
                    });
                }
            });
        });
        const uint64_t gw = (uint64_t)tile * 512u +
                            ((lane & 1u) | ((lane >> 5) << 1) | (((lane >> 1) & 1u) << 2) | (wave << 3) | (((lane >> 2) & 7u) << 6));
        if (gw < a.W) {
            uint64_t *dst = static_cast<uint64_t *>(a.dst) + slot * a.dst_stride + gw;
#pragma unroll
            for (int p = 0; p < 8; ++p)
                if ((uint32_t)p < a.planes) dst[(uint64_t)p * a.W] = ((uint64_t)hi[p] << 32) | lo[p];
        }
    } else if constexpr (OUT == OUT_PACK && DITHER && !STATS) {
        // Def. 3.2 with the dither u = (2 r + 1 - 2^24) 2^-24, r the top 24 bits of the 32-bit draw w:
        //   z + lambda' u >= 0  <=>  r >= ((2^24 - 1) - z 2^24 / lambda') / 2  <=>  w >= T,  T = 2^31 - 128 - 128 z 2^24 / lambda',
        // so a coordinate costs one multiply-add, one saturating conversion (T <= 0 -> 0: always +1; T >= 2^32 -> 2^32 - 1)
        // and one integer compare.  T is rounded to 256 (1 in r), i.e. the threshold moves by at most lambda' 2^-24, a
        // hundred times below the near-tie margin.  A NaN amplitude gives all bits 0, as NaN comparisons do.
        uint32_t my_lo = 0u, my_hi = 0u;
        static_for<16>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            uint32_t w[4];
            const uint32_t lg = local_of(2 * g); // b6 = b7 = 0
            philox((uint32_t)(((base + lg) >> 8) << 6) | lane, key_dit, w);
            float kq_g = 0.f;
            if constexpr (!SMALLB) kq_g = lam[lg >> S];
            uint64_t word[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int r = 2 * g + (s & 1) + 32 * (s >> 1); // slot s = b6 | b7 << 1
                float kq = kq_g;
                if constexpr (SMALLB) kq = lam[local_of(r) >> S];
                uint32_t thr;
                asm("v_cvt_u32_f32 %0, %1" : "=v"(thr) : "v"(fmaf(v[r], kq, 2147483520.f)));
                word[s] = __ballot(w[s] >= thr) & __ballot(kq == kq);
            }
            // the 64-bit word of register r goes to lane r: one write into that lane per half
            static_for<4>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                constexpr int r = 2 * g + (s & 1) + 32 * (s >> 1);
                my_lo = write_lane<r>(my_lo, (uint32_t)word[s]);
                my_hi = write_lane<r>(my_hi, (uint32_t)(word[s] >> 32));
            });
        });
        // lane j holds the word of register j
        const uint64_t gw = (uint64_t)tile * 512u +
                            ((lane & 1u) | ((lane >> 5) << 1) | (((lane >> 1) & 1u) << 2) | (wave << 3) | (((lane >> 2) & 7u) << 6));
        if (gw < a.W)
            static_cast<uint64_t *>(a.dst)[slot * a.dst_stride + gw] = ((uint64_t)my_hi << 32) | my_lo;
    } else if constexpr (OUT == OUT_PACK) {
        uint32_t my_lo = 0u, my_hi = 0u;
        const float tscale = a.sqrtb * 5.9604644775390625e-08f; // 2^-24: u = m * 2^-24 with m odd
        static_for<16>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            uint32_t w[4] = { 0u, 0u, 0u, 0u };
            const uint32_t lg = local_of(2 * g); // b6 = b7 = 0
            float thr_g = 0.f;
            if constexpr (DITHER) {
                philox((uint32_t)(((base + lg) >> 8) << 6) | lane, key_dit, w);
                if constexpr (!SMALLB) thr_g = lam[lg >> S] * tscale;
            }
            uint64_t word[4];
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int r = 2 * g + (s & 1) + 32 * (s >> 1); // slot s = b6 | b7 << 1
                float tv = v[r];
                if constexpr (DITHER) {
                    float thr = thr_g;
                    if constexpr (SMALLB) thr = lam[local_of(r) >> S] * tscale;
                    // m = 2 r + 1 - 2^24 for the 24-bit draw r; both conversions are exact
                    const float m = fmaf((float)(w[s] >> 8), 2.f, -16777215.f);
                    tv = fmaf(thr, m, tv);
                }
                word[s] = __ballot(tv >= 0.f);
            }
            // the 64-bit word of register r goes to lane r: one write into that lane per half
            static_for<4>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                constexpr int r = 2 * g + (s & 1) + 32 * (s >> 1);
                my_lo = write_lane<r>(my_lo, (uint32_t)word[s]);
                my_hi = write_lane<r>(my_hi, (uint32_t)(word[s] >> 32));
            });
        });
        // lane j holds the word of register j
        const uint64_t gw = (uint64_t)tile * 512u +
                            ((lane & 1u) | ((lane >> 5) << 1) | (((lane >> 1) & 1u) << 2) | (wave << 3) | (((lane >> 2) & 7u) << 6));
        if (gw < a.W)
            static_cast<uint64_t *>(a.dst)[slot * a.dst_stride + gw] = ((uint64_t)my_hi << 32) | my_lo;
    } else if constexpr (OUT == OUT_I16) {
        // pairs (b0 = 0, 1) packed into one dword; a wave writes 256 contiguous bytes per register pair
        uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<int16_t *>(a.dst) + slot * a.dst_stride + base);
#pragma unroll
        for (int r = 0; r < kV; r += 2) {
            // dword index = coordinate / 2 = lane | b7 << 6 | b8 << 7 | wave << 8 | (b12..b14) << 11
            const uint32_t di = lane | ((uint32_t)(r >> 5) << 6) | ((uint32_t)((r >> 1) & 1) << 7) | (wave << 8) |
                                ((uint32_t)((r >> 2) & 7) << 11);
            dst[di] = __builtin_amdgcn_perm((uint32_t)v[r + 1], (uint32_t)v[r], 0x05040100u);
        }
    } else if constexpr (OUT == OUT_I32) {
        int32_t *dst = static_cast<int32_t *>(a.dst) + slot * a.dst_stride + base;
#pragma unroll
        for (int r = 0; r < kV; ++r) dst[local_of(r)] = v[r];
    } else {
        float *dst = static_cast<float *>(a.dst);
#pragma unroll
        for (int r = 0; r < kV; ++r) {
            const uint32_t loc = local_of(r);
            const uint64_t i = base + loc;
            const uint32_t ew = epsw[wave * 128u + (((r & 31) >> 1) | ((r >> 5) << 4)) * 4 + ((r & 1) << 1) + (lane >> 5)];
            const float val = flip_if((lam[loc >> S] * a.out_coef) * (float)v[r], (ew >> (lane & 31u)) & 1u);
            if (i < a.len_out) {
                if (a.store_mode == STORE_SET) dst[i] = val;
                else if (a.store_mode == STORE_ACC) dst[i] += val;
                else dst[i] -= a.delta * val;
            }
        }
    }
}

template <int IN, int OUT, bool DITHER = false, bool SMALLB = false, int SC = 0, bool MULTIK = false, bool STATS = false,
          bool GUARDED = true>
__global__ __launch_bounds__(kThreads, 4) void k_contig(const ContigArgs a, const PtrTab tab)
{
    __shared__ uint32_t lds[kLdsWords];
    contig_tile<IN, OUT, DITHER, SMALLB, SC, MULTIK, STATS, false, GUARDED>(a, tab, a.tile0 + blockIdx.x, blockIdx.y, lds, threadIdx.x);
}

// Encode of blocks of exactly 2^16 coordinates in one pass: 1024 threads, one block (two tiles) per workgroup.
template <bool DITHER, bool MULTIK, bool GUARDED = true>
__global__ __launch_bounds__(2 * kThreads) void k_contig_pair(const ContigArgs a, const PtrTab tab)
{
    __shared__ uint32_t lds[2 * kLdsWords];
    const uint32_t h = threadIdx.x >> 9;
    contig_tile<IN_GRAD, OUT_PACK, DITHER, false, 15, MULTIK, false, true, GUARDED>(a, tab, a.tile0 + 2u * blockIdx.x + h, blockIdx.y, lds + h * kLdsWords,
                                                                           threadIdx.x & 511u, lds + (h ^ 1u) * kLdsWords);
}

} // namespace fo
