// Decode-side low stages straight from the packed sign bits: the fifteen Walsh-Hadamard stages of
// every 2^15-coordinate tile of H^T q (Def. 3.8), q in {-1,+1}^n given as bits, result as int16.
//
// The data are small integers, which buys two things over the generic tile kernel:
//   * the five stages on b0..b4 act on the 32 signs of one packed 32-bit word, and output j of that
//     32-point transform is sum_i W_j(i) (2 c_i - 1) = 2 popcount(word ^ mask_j) - 32, where mask_j has
//     bit i set when popcount(i & j) is odd: one xor and one bit count per output instead of an unpack
//     and five additions;
//   * every later stage adds or subtracts whole registers, so two int16 values ride in one register
//     (the pair b0 = 0, 1, which is also the pair the int16 intermediate stores in one dword) and one
//     packed add serves two butterflies.
// As everywhere on the decode side the values are carried divided by two: popcount - 16 instead of
// 2 popcount - 32, so the result of all fifteen stages fits int16 exactly.  The -16 is not applied per
// value: a constant offset of 16 on every input of the remaining ten stages ends up as 16 * 2^10 on the
// coordinates whose bits b5..b14 are all zero and nowhere else, and is taken off there at the end
// (int16 arithmetic wraps, so the detour through the offset cannot lose anything; the library is built with
// -fwrapv, which makes that wrap-around defined behaviour of the signed vector types).
//
// Index-bit choreography (dword = pair of coordinates, bits b1..b14):
//   LA: regs = (b1,b2,b3,b4,b11)   lanes = (b5..b10)            waves = (b12,b13,b14)   stages b0..b4, b11
//   LB: regs = (b5..b9)            lanes = (b1,b2,b3,b4,b11,b10)                        stages b5..b9, b10 (lane swap)
//   LC: regs = (b12,b13,b14,b7,b8) lanes = (b1..b6)             waves = (b9,b10,b11)    stages b12,b13,b14
#pragma once
#include "fo_contig.h"

namespace fo {

typedef short s16x2 __attribute__((ext_vector_type(2)));

constexpr uint32_t walsh_mask32(int j)
{
    uint32_t m = 0;
    for (int i = 0; i < 32; ++i)
        if (__builtin_popcount((unsigned)(i & j)) & 1) m |= 1u << i;
    return m;
}

// Decode-side stages of one tile from its 1024 packed 32-bit words, result in layout LC as 32 packed pairs.
// SC = 15: all fifteen stages (transform length >= 2^15); SC = 0: the S = 6..15 stages of a blocked transform,
// S read at run time (stage k runs iff k < S; the popcount stages b0..b4 always do); other SC: compiled for S = SC.
// words points at the party's packed vector.
// xa, xb: kXWords words of LDS each for the first (wave-private) and the second (workgroup-wide) exchange; they
// may be the same buffer.  The second exchange starts with a barrier (all earlier reads of xb are over) and its
// reads are not followed by one: a caller that loops must not write xb again before its next barrier, which a
// second call does by itself when xa and xb differ.
// declow_front: up to the point where the tile sits in xb in layout LB and the barrier after it has been passed;
// declow_back: the read into layout LC and the last three stages.  declow_tile is the two in a row.
template <int SC>
__device__ __forceinline__ void declow_front(const uint32_t *words, uint64_t W, uint32_t tile, uint32_t S_arg, uint32_t *xa,
                                             uint32_t *xb, s16x2 (&v)[32], const uint32_t t)
{
    const uint32_t lane = t & 63u, wave = t >> 6;
    const uint32_t S = SC ? (uint32_t)SC : S_arg;

    // ------------------------------------------------------------------ stages b0..b4 (layout LA)
#pragma unroll
    for (int x = 0; x < 2; ++x) {
        const uint64_t gh = (uint64_t)tile * 1024u + wave * 128u + x * 64u + lane; // 32-bit half word
        const uint32_t w = (gh < 2 * W) ? words[gh] : 0u;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t hi = (uint32_t)__builtin_popcount(w ^ walsh_mask32(2 * k + 1));
            const uint32_t both = (uint32_t)__builtin_popcount(w ^ walsh_mask32(2 * k)) + (hi << 16);
            v[x * 16 + k] = __builtin_bit_cast(s16x2, both);
            // blocked transforms take the popcount's offset off here; the full-tile case does it at the end
            if constexpr (SC != 15) v[x * 16 + k] -= s16x2{ 16, 16 };
        }
    }
    if (S > 11u) bfly<s16x2, 4, 32>(v); // b11

    // ------------------------------------------------------------------ exchange LA -> LB (inside each half wave)
    {
        uint32_t *const wb = xa + wave * 2112u + (lane >> 5) * 1056u;
        const uint32_t col = lane & 31u;
#pragma unroll
        for (int r = 0; r < 32; ++r) wb[r * 33 + col] = __builtin_bit_cast(uint32_t, v[r]);
        wave_sync();
#pragma unroll
        for (int r = 0; r < 32; ++r) v[r] = __builtin_bit_cast(s16x2, wb[col * 33 + r]);
    }
    bfly<s16x2, 0, 32>(v); // b5: every transform has at least 2^6 points
    if (S > 6u) bfly<s16x2, 1, 32>(v);
    if (S > 7u) bfly<s16x2, 2, 32>(v);
    if (S > 8u) bfly<s16x2, 3, 32>(v);
    if (S > 9u) bfly<s16x2, 4, 32>(v);
    if (S > 10u) bfly_lane5<s16x2, 32>(v); // b10

    // ------------------------------------------------------------------ exchange LB -> LC (whole workgroup)
    // Address = dword index D plus 16 words of padding per 1024: the writers' lanes spread over
    // (b1..b4) and b11 (D bit 10), the readers' over (b1..b6).
    __syncthreads(); // every wave is done with its part of the first exchange
    {
        const uint32_t b11 = (lane >> 4) & 1u, b10 = lane >> 5;
        const uint32_t wofs = (lane & 15u) + b10 * 512u + b11 * 1024u + wave * 2048u + 16u * (b11 + 2u * wave);
#pragma unroll
        for (int r = 0; r < 32; ++r) xb[wofs + r * 16] = __builtin_bit_cast(uint32_t, v[r]);
    }
    __syncthreads();
}

template <int SC>
__device__ __forceinline__ void declow_back(const uint32_t *xb, uint32_t S_arg, s16x2 (&v)[32], const uint32_t t)
{
    const uint32_t lane = t & 63u, wave = t >> 6;
    const uint32_t S = SC ? (uint32_t)SC : S_arg;
    {
        const uint32_t rofs = lane + wave * 256u + 16u * (wave >> 2);
#pragma unroll
        for (int r = 0; r < 32; ++r) // register r = (b12,b13,b14,b7,b8)
            v[r] = __builtin_bit_cast(s16x2, xb[rofs + ((r >> 3) & 1) * 64 + (r >> 4) * 128 + (r & 7) * (2048 + 32)]);
    }
    if (S > 12u) bfly<s16x2, 0, 32>(v);
    if (S > 13u) bfly<s16x2, 1, 32>(v);
    if (S > 14u) bfly<s16x2, 2, 32>(v);

    // the popcount offset, gathered by the ten later stages on the coordinates with b5..b14 = 0
    if constexpr (SC == 15)
        if (t < 16u) v[0] -= s16x2{ 16384, 16384 };
}

template <int SC>
__device__ __forceinline__ void declow_tile(const uint32_t *words, uint64_t W, uint32_t tile, uint32_t S_arg, uint32_t *xa,
                                            uint32_t *xb, s16x2 (&v)[32], const uint32_t t = threadIdx.x)
{
    // t: the thread index; a caller that loops may pass a copy the compiler cannot see through, so that the
    // offsets derived from it are recomputed per call instead of being kept in registers across the loop
    declow_front<SC>(words, W, tile, S_arg, xa, xb, v, t);
    declow_back<SC>(xb, S_arg, v, t);
}

// The back half for transforms of exactly 2^16 points, where two groups of 512 threads in one workgroup hold the
// two tiles of a block (UPPER: the group with the upper tile).  Both have run declow_front<15>; xb_own and xb_oth
// are their exchange buffers.  The sixteenth stage, on bit 15, pairs dword D of the lower tile with dword D of
// the upper one, and it is done here, before the stages on b12..b14 (stages commute): each group reads both
// buffers and keeps lo + hi (lower) or lo - hi (upper).  The results of all sixteen stages need 17 bits (half
// values of up to 2^16 signs), so the last stage, b14, runs on int32; up to there packed int16 is exact (it
// wraps, but every true value before the last stage fits).  Eight packed registers at a time: register group
// G = (b7,b8) holds the registers r = q + 8 G, q = (b12,b13,b14), and emit(G, w) gets their values as
// w[2 q + j], j = b0.  The popcount offset of 16 per input has grown to 16 * 2^10 on the coordinates with
// b5..b13 = 0 of the lower tile before the last stage (it cancels in the upper tile) and is taken off there.
template <bool UPPER, typename F>
__device__ __forceinline__ void declow_pair_back(const uint32_t *xb_own, const uint32_t *xb_oth, const uint32_t t, F &&emit)
{
    const uint32_t lane = t & 63u, wave = t >> 6;
    const uint32_t rofs = lane + wave * 256u + 16u * (wave >> 2);
    static_for<4>([&](auto G) {
        s16x2 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint32_t off = rofs + (G.value & 1) * 64 + (G.value >> 1) * 128 + q * (2048 + 32);
            const s16x2 a = __builtin_bit_cast(s16x2, xb_own[off]), b = __builtin_bit_cast(s16x2, xb_oth[off]);
            v[q] = UPPER ? b - a : a + b; // b15
        }
        bfly<s16x2, 0, 8>(v); // b12
        bfly<s16x2, 1, 8>(v); // b13
        if (!UPPER && G.value == 0 && t < 16u) {
            v[0] -= s16x2{ 16384, 16384 };
            v[4] -= s16x2{ 16384, 16384 };
        }
        int32_t w[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) { // b14
            const s16x2 a = v[q], b = v[q + 4];
            w[2 * q] = (int32_t)a.x + (int32_t)b.x;
            w[2 * q + 1] = (int32_t)a.y + (int32_t)b.y;
            w[2 * (q + 4)] = (int32_t)a.x - (int32_t)b.x;
            w[2 * (q + 4) + 1] = (int32_t)a.y - (int32_t)b.y;
        }
        emit(G, w);
    });
}

// dword index (= coordinate / 2) inside the tile of register r of this thread in layout LC
__device__ __forceinline__ constexpr uint32_t declow_reg_dword(int r)
{
    return ((uint32_t)((r >> 3) & 1) << 6) | ((uint32_t)(r >> 4) << 7) | ((uint32_t)(r & 7) << 11);
}

// (Kernels that are not templates are static: these headers are included by several translation units.)
// Uses src, src_stride (64-bit words between slots), dst, dst_stride (int16 elements between slots) and W
// of the argument block; the transform length is at least 2^15, so every tile is complete.
static __global__ __launch_bounds__(kThreads, 4) void k_declow(const ContigArgs a)
{
    __shared__ uint32_t xbuf[kXWords];
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x, slot = blockIdx.y;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(static_cast<const uint64_t *>(a.src) + slot * a.src_stride);
    s16x2 v[32];
    declow_tile<15>(src, a.W, tile, 15u, xbuf, xbuf, v);

    // store: a wave writes 256 contiguous bytes per register
    uint32_t *dst = reinterpret_cast<uint32_t *>(static_cast<int16_t *>(a.dst) + slot * a.dst_stride + ((uint64_t)tile << kTileLog2) + (uint64_t)tile * a.dst_pad);
    const uint32_t dt = lane | (wave << 8);
#pragma unroll
    for (int r = 0; r < 32; ++r) dst[dt + declow_reg_dword(r)] = __builtin_bit_cast(uint32_t, v[r]);
}

} // namespace fo
