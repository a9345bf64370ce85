// Decode-side transform of a 2^15-coordinate tile on the matrix cores (transform lengths 2^6 .. 2^15, whole or
// blocked): H^T q for q in {-1,+1}^b given as packed bits (Def. 3.8), as three small dense +-1 matrix products.
//
// The tile-local coordinate i = (b0..b14) is split as (b0..b5 | b6..b10 | b11..b14) and the transform, a
// Kronecker product of 2x2 blocks, factors along the same split:
//   stage 1, b0..b5 : v_mfma_scale_f32_32x32x64_f8f6f4 with both operands in fp4 (E2M1).  A row of the data
//                     operand is one 64-coordinate group, whose sign bits are turned into fp4 digits without any
//                     unpacking: `w & 0x11111111` is eight fp4 values 0.5 * bit, `w & 0x22222222` eight values
//                     1.0 * bit, `w & 0x44444444` eight values 2.0 * bit (the fourth bit of each nibble, which
//                     would be a sign bit, is shifted down first).  The constant operand holds the matching
//                     entries of H_64 divided by those weights (+-2, +-1, +-0.5: all fp4 numbers).  With bits
//                     c in {0,1} instead of signs q = 2c - 1 the product is (H^T q)/2 + 32 [t = 0]: the decode
//                     side carries half values anyway, and the constant rides along on the zero-frequency
//                     coordinate of every block (it grows to 2^(S-1) there) and is taken off at the end.
//   stage 2, b6..b10: two v_mfma_f32_32x32x16_f16.  Inputs are integers of magnitude <= 64, exact in fp16.
//   stage 3, b11..b14 and b5 as a bystander: two more, on integers <= 2048 (still exact in fp16; the fp32
//                     accumulators are exact to 2^24).
// Blocked transforms shorter than the tile use the same code: the constant operand of a stage is the Kronecker
// product of 2x2 Hadamard blocks on the index bits below log2 b and 2x2 identities on the others.
//
// The data always enter as the A operand, rows = an index that is not being transformed, k = the one that is.
// The result D[row][col] then has the transformed index on the lanes and the old rows in the registers, i.e.
// each product also transposes, and the next stage can contract over the registers again with no data movement
// (the constant operands are permuted to the order in which the previous result's registers hold the rows).
// Only between stages 2 and 3 do values cross waves: through LDS, as packed fp16 pairs (b0 = 0, 1), and b0 goes
// through stage 3 as a bystander (identity) next to b11..b14, so that its contraction has 32 terms.
//
// 1024 threads; wave w handles the slab b11..b14 = w in stages 1 and 2 and the columns b6..b10 = 2w, 2w+1 in stage 3.
// After stage 3 lane (j, h) (j = lane % 32, h = lane / 32) holds in register r of column group gi the coordinate
//   b0 = j & 1, (b1, b2) = r & 3, b3 = h, b4 = (r >> 2) & 1, b5 = r >> 3, b6..b10 = 2w + gi, b11..b14 = j >> 1:
// the sixteen values of a group lie in two neighbouring 32-coordinate eps words and in one block.
#pragma once
#include "fo_contig.h"

namespace fo {

typedef int mf_v8i __attribute__((ext_vector_type(8)));
typedef float mf_v16f __attribute__((ext_vector_type(16)));
typedef _Float16 mf_v8h __attribute__((ext_vector_type(8)));

constexpr uint32_t kMfThreads = 1024;
constexpr uint32_t kMfRowBytes = 2064;           // 32 columns (b6..b10) of 64 bytes per row (b1..b5), padded by 16
constexpr uint32_t kMfXBytes = 32u * kMfRowBytes; // one exchange buffer
constexpr uint32_t kMfXWords = kMfXBytes / 4u;
// eps table of a tile (1024 words, word e covers coordinates 32 e ..): after stage 3 the 32 lanes of a half wave
// read words 64 apart, so every 64 words are followed by 4 words of padding
constexpr uint32_t kMfEpsWords = 16u * 68u;
__device__ __forceinline__ uint32_t mf_eps_pos(uint32_t e) { return e + 4u * (e >> 6); }

__device__ __forceinline__ uint32_t parity32(uint32_t x) { return (uint32_t)__builtin_popcount(x) & 1u; }

// Constant operands of the three stages for this lane (wave-dependent only through the stage-3 swizzle).
struct MfConst {
    uint32_t b1[4];   // stage 1, fp4, outputs t = 0..31; outputs 32..63 flip every sign where lane / 32 = 1 (b1flip)
    uint32_t b1flip;
    mf_v8h b2[2];
    mf_v8h b3[2];
};

// S = log2 of the transform length (6..15); wave = index of the wave in the workgroup (0..15).
__device__ __forceinline__ void mf_build_constants(MfConst &k, uint32_t S, uint32_t lane, uint32_t wave)
{
    const uint32_t col = lane & 31u, hb = lane >> 5;
    // stage 1: entry for k = 32 hb + 8 q + nib is H_64[32 hb + 4 nib + q][t] / (0.5, 1, 2, 2)[q], t = 32 m + col;
    // the sign is parity((4 nib + q) & col) ^ (hb & m)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t mag = q == 0 ? 4u : q == 1 ? 2u : 1u; // fp4 codes of 2.0, 1.0, 0.5
        uint32_t d = 0;
#pragma unroll
        for (int nib = 0; nib < 8; ++nib) d |= (mag | (parity32((4u * nib + q) & col) << 3)) << (4 * nib);
        k.b1[q] = d;
    }
    k.b1flip = hb ? 0x88888888u : 0u;
    // stage 2: rows g = b6..b10 in the order the stage-1 result's registers hold them
    const uint32_t tr2 = S >= 11u ? 31u : ((1u << (S - 6u)) - 1u), id2 = 31u & ~tr2;
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t g = 8u * (2u * mm + (e >> 2)) + 4u * hb + (e & 3u);
            const float v = ((g ^ col) & id2) ? 0.f : (parity32(g & col & tr2) ? -1.f : 1.f);
            k.b2[mm][e] = (_Float16)v;
        }
    // stage 3: k = (slab, b0) in the order the exchange buffer delivers it to this wave; column = (b0, b11..b14)
    const uint32_t tr3 = S <= 11u ? 0u : ((1u << (S - 11u)) - 1u), id3 = 15u & ~tr3;
    const uint32_t s = wave >> 1;
    const uint32_t sg2 = col >> 1, m2 = col & 1u;
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t sg = (4u * (2u * mm + hb) + (e >> 1)) ^ s, mb = e & 1u;
            const float v = (mb != m2 || ((sg ^ sg2) & id3)) ? 0.f : (parity32(sg & sg2 & tr3) ? -1.f : 1.f);
            k.b3[mm][e] = (_Float16)v;
        }
}

__device__ __forceinline__ uint32_t mf_pack(float lo, float hi)
{
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(lo, hi)); // integers below 2^11: exact
}

// Stages 1 and 2 of this wave's slab from its lanes' packed word, and the write into the exchange buffer.
// xw: this lane's write base (bytes) inside the buffer.  After stage 2 register r of the product for b5 = m holds
// b0..b4 = 8 (r / 4) + 4 h + r % 4: registers 2u, 2u + 1 are a pair b0 = 0, 1 and go to row (b1..b4, b5) as one dword.
__device__ __forceinline__ void mf_front(uint32_t w, const MfConst &k, char *xbuf, uint32_t xw)
{
    const mf_v8i a = { (int)(w & 0x11111111u), (int)(w & 0x22222222u), (int)(w & 0x44444444u), (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0 };
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint32_t f = m ? k.b1flip : 0u;
        const mf_v8i b = { (int)(k.b1[0] ^ f), (int)(k.b1[1] ^ f), (int)(k.b1[2] ^ f), (int)(k.b1[3] ^ f), 0, 0, 0, 0 };
        const mf_v16f z = { 0 };
        const mf_v16f d1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, z, 4, 4, 0, 127, 0, 127);
        uint32_t pk[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) pk[u] = mf_pack(d1[2 * u], d1[2 * u + 1]);
        const mf_v8h p0 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&pk[0]));
        const mf_v8h p1 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&pk[4]));
        mf_v16f e = __builtin_amdgcn_mfma_f32_32x32x16_f16(p0, k.b2[0], z, 0, 0, 0);
        e = __builtin_amdgcn_mfma_f32_32x32x16_f16(p1, k.b2[1], e, 0, 0, 0);
#pragma unroll
        for (int u = 0; u < 8; ++u) // row (b1..b4 | b5) = 4 (u / 2) + 2 h + u % 2 + 16 m; the lane part is in xw
            *reinterpret_cast<uint32_t *>(xbuf + xw + (4u * (u >> 1) + (u & 1u) + 16u * m) * kMfRowBytes) = mf_pack(e[2 * u], e[2 * u + 1]);
    }
}

// Stage 3 for one row group: reads this lane's two 16-byte pieces at xr (bytes) and returns the sixteen half values
// (H^T q)_i / 2 (+ 2^(S-1) on the first coordinate of every block), i as given in the header comment.
__device__ __forceinline__ mf_v16f mf_back(const mf_v8h (&b3)[2], const char *xbuf, uint32_t xr)
{
    const mf_v8h a0 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(xbuf + xr));
    const mf_v8h a1 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(xbuf + xr + 32u));
    mf_v16f z = { 0 };
    mf_v16f d = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, b3[0], z, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, b3[1], d, 0, 0, 0);
}

// ---------------------------------------------------------------------------------------------
// Transforms of exactly 2^16 points (a block of two tiles): split (b0..b5 | b6..b10 | b11..b15), all three stages
// full Hadamard products.  Two workgroups share a block: both run stages 1 and 2 on all 32 slabs (the packed
// signs are small, reading and transforming them twice is cheap), but workgroup q keeps only the columns
// b10 = q, so each holds 2^15 accumulators, as for a single tile.  Wave w handles the slabs b11..b15 = 2w, 2w + 1
// and pairs them in one dword, so that the stage-3 contraction index (the slab) is contiguous in LDS.
// After stage 3 lane (j, h) holds in register r of column group g = (b5 | b6..b9) the coordinate
//   b0..b4 = 8 (r / 4) + 4 h + r % 4, b5 = g / 16, b6..b9 = g % 16, b10 = q, b11..b15 = j:
// sixteen values of one eps word.
// ---------------------------------------------------------------------------------------------
constexpr uint32_t kMf16EpsWords = 32u * 36u; // eps words of one workgroup's half block: 32 per slab, padded to 36
__device__ __forceinline__ uint32_t mf16_eps_pos(uint32_t low5, uint32_t slab) { return low5 + 36u * slab; }

struct MfConst16 {
    uint32_t b1[4];
    uint32_t b1flip;
    mf_v8h b2[2];
    mf_v8h b3[2];
};

__device__ __forceinline__ void mf16_build_constants(MfConst16 &k, uint32_t lane, uint32_t wave)
{
    const uint32_t col = lane & 31u, hb = lane >> 5;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t mag = q == 0 ? 4u : q == 1 ? 2u : 1u;
        uint32_t d = 0;
#pragma unroll
        for (int nib = 0; nib < 8; ++nib) d |= (mag | (parity32((4u * nib + q) & col) << 3)) << (4 * nib);
        k.b1[q] = d;
    }
    k.b1flip = hb ? 0x88888888u : 0u;
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t g = 8u * (2u * mm + (e >> 2)) + 4u * hb + (e & 3u);
            k.b2[mm][e] = (_Float16)(parity32(g & col) ? -1.f : 1.f);
        }
    // stage 3: k = slab in the order the exchange buffer delivers it to this wave (dwords swizzled by f), column = slab'
    const uint32_t f = (wave & 7u) >> 1;
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t sg = 2u * ((4u * (2u * mm + hb) + (e >> 1)) ^ f) + (e & 1u);
            k.b3[mm][e] = (_Float16)(parity32(sg & col) ? -1.f : 1.f);
        }
}

// Stages 1 and 2 of this wave's two slabs (packed words w0, w1 of this lane) and the write into the exchange buffer:
// row b0..b4, column group (b5 | b6..b9), dword = wave (swizzled by the column group), halves = the two slabs.
// keep: this lane's column b6..b10 belongs to the workgroup's half (b10 = q).
__device__ __forceinline__ void mf16_front(uint32_t w0, uint32_t w1, const MfConst16 &k, char *xbuf, uint32_t xw, bool keep)
{
    const mf_v16f z = { 0 };
    const uint32_t ws[2] = { w0, w1 };
#pragma unroll
    for (int m = 0; m < 2; ++m) {
        const uint32_t f = m ? k.b1flip : 0u;
        const mf_v8i b = { (int)(k.b1[0] ^ f), (int)(k.b1[1] ^ f), (int)(k.b1[2] ^ f), (int)(k.b1[3] ^ f), 0, 0, 0, 0 };
        mf_v16f e[2];
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            const uint32_t w = ws[sl];
            const mf_v8i a = { (int)(w & 0x11111111u), (int)(w & 0x22222222u), (int)(w & 0x44444444u), (int)((w >> 1) & 0x44444444u), 0, 0, 0, 0 };
            const mf_v16f d1 = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, z, 4, 4, 0, 127, 0, 127);
            uint32_t pk[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) pk[u] = mf_pack(d1[2 * u], d1[2 * u + 1]);
            const mf_v8h p0 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&pk[0]));
            const mf_v8h p1 = __builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&pk[4]));
            e[sl] = __builtin_amdgcn_mfma_f32_32x32x16_f16(p0, k.b2[0], z, 0, 0, 0);
            e[sl] = __builtin_amdgcn_mfma_f32_32x32x16_f16(p1, k.b2[1], e[sl], 0, 0, 0);
        }
        if (keep) {
#pragma unroll
            for (int r = 0; r < 16; ++r) // row b0..b4 = 8 (r / 4) + 4 h + r % 4 (lane part in xw); column group + 16 m
                *reinterpret_cast<uint32_t *>(xbuf + xw + (8u * (r >> 2) + (r & 3u)) * kMfRowBytes + 16u * 64u * m) = mf_pack(e[0][r], e[1][r]);
        }
    }
}

} // namespace fo
