// Strided-tile kernel: up to ten Walsh-Hadamard stages on index bits above the contiguous tile
// (transform lengths above 2^15).  A tile is R = 2^hb rows by 2^(15-hb) consecutive columns, rows
// 2^ls coordinates apart; the stages act along the rows' axis only.  Global accesses are one
// dword per lane with at least 32 consecutive coordinates (128 B) per row segment.
//
// Tile coordinate u = row << cb | col (cb = 15 - hb).
//   LA (loads):              lanes = (u0..u5)     waves = (u6,u7,u8)     regs = (u9..u14)
//   LB (after the exchange): lanes = (u0..u4,u9)  waves = (u10,u11,u12)  regs = (u5,u6,u7,u8,u13,u14)
// Modes
//   SM_ENC_FIRST : fp32 gradient (zero padded), eps flip on load, tile sum of squares -> fp32 intermediate
//   SM_DEC_LAST  : int32 intermediate -> lambda/sqrt(b) scaling, eps flip, store / SGD update (Def. 3.8)
//   SM_MID       : intermediate in, intermediate out (three-pass transforms)
//   SM_SERVER    : for every worker: int32 intermediate -> remaining inverse stages, scale, flip,
//                  accumulate the mean (eq. "server average"); then eps^s flip and the forward
//                  stages of the re-encode (Sec. 4, server-to-workers encoding) -> fp32 intermediate
#pragma once
#include "fo_contig.h"

namespace fo {

enum { SM_ENC_FIRST = 0, SM_DEC_LAST = 1, SM_MID_F32 = 2, SM_MID_I32 = 3, SM_SERVER = 4 };

struct StridedArgs {
    const void *src;       // fp32 / int32 [slot][ntot] (ENC_FIRST: gradients, or pointer table)
    uint64_t src_stride;
    void *dst;             // fp32 / int32 [slot][ntot]; DEC_LAST: fp32 [len_out]
    uint64_t dst_stride;
    const float *scales;   // [slot or worker][nblocks]
    uint64_t scales_stride;
    float *partials;       // ENC_FIRST: [slot][ntiles] tile sums of squares
    float *gbar;           // SERVER: optional fp32 [ntot] copy of the mean
    uint64_t len_in, len_out;
    uint32_t ls, hb;       // log2 row stride, number of stages (1..10)
    uint32_t logb;
    uint32_t use_tab;
    uint32_t M;            // SERVER: workers to accumulate
    uint32_t store_mode;
    uint32_t eps_party0;
    uint32_t k0, k1, round_lo;
    float out_coef;        // 1/sqrt(b) (times 1/M in SERVER)
    float delta;
};

// Element offset of tile coordinate u from the tile origin.  Each bit of u has a fixed weight
// (column bits keep theirs, row bits move up to the row stride), so off(u1 | u2) = off(u1) + off(u2)
// for disjoint bit sets: a thread adds its own part once and a wave-uniform part per register.
struct StridedGeom {
    uint64_t origin; // coordinate of u = 0
    uint32_t cb, ls;
    __device__ __forceinline__ uint32_t off(uint32_t u) const
    {
        return ((u >> cb) << ls) + (u & ((1u << cb) - 1u));
    }
};

// thread part and register part of a tile coordinate in the two layouts
__device__ __forceinline__ uint32_t ua_thread(uint32_t lane, uint32_t wave) { return lane | (wave << 6); }
__device__ __forceinline__ constexpr uint32_t ua_reg(int r) { return (uint32_t)r << 9; }
__device__ __forceinline__ uint32_t ub_thread(uint32_t lane, uint32_t wave)
{
    return (lane & 31u) | ((lane >> 5) << 9) | (wave << 10);
}
__device__ __forceinline__ constexpr uint32_t ub_reg(int r)
{
    return ((uint32_t)(r & 1) << 5) | ((uint32_t)((r >> 1) & 7) << 6) | ((uint32_t)(r >> 4) << 13);
}

// eps words of the tile, one 32-bit word per group of 32 consecutive columns (u >> 5)
__device__ __forceinline__ void fill_eps(uint32_t *epsw, const StridedGeom &g, const RngKey &key, uint32_t t)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const uint32_t grp = t + h * kThreads;
        const uint64_t i = g.origin + g.off(grp << 5);
        uint32_t w[4];
        philox((uint32_t)(i >> 7), key, w);
        const uint32_t sel = (uint32_t)(i >> 5) & 3u;
        epsw[grp] = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
    }
}

template <typename T>
__device__ __forceinline__ void stages_a(T (&v)[kV], uint32_t cb) // LA registers hold u9..u14
{
    if (cb <= 9u) bfly<T, 0>(v);
    if (cb <= 10u) bfly<T, 1>(v);
    if (cb <= 11u) bfly<T, 2>(v);
    if (cb <= 12u) bfly<T, 3>(v);
    if (cb <= 13u) bfly<T, 4>(v);
    bfly<T, 5>(v);
}
template <typename T>
__device__ __forceinline__ void stages_b(T (&v)[kV], uint32_t cb) // LB registers 0..3 hold u5..u8
{
    if (cb <= 5u) bfly<T, 0>(v);
    if (cb <= 6u) bfly<T, 1>(v);
    if (cb <= 7u) bfly<T, 2>(v);
    if (cb <= 8u) bfly<T, 3>(v);
}

// LA -> LB (forward) or LB -> LA (!forward) through LDS, two halves split on register bit 5 (u14).
// Word address bits: 0-4 u0..u4 | 5 u5^u9 | 6 u9 | 7-9 u10..u12 | 10-12 u6..u8 | 13 u13.
template <typename T, bool FORWARD>
__device__ __forceinline__ void exchange(T (&v)[kV], uint32_t *xbuf, uint32_t lane, uint32_t wave)
{
    const uint32_t l5 = lane >> 5, lo = lane & 31u;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
        if (sub) __syncthreads();
        if (FORWARD) {
#pragma unroll
            for (int r = 0; r < 32; ++r) // LA register r = (u9..u13)
                xbuf[lo | ((l5 ^ (uint32_t)(r & 1)) << 5) | ((uint32_t)(r & 15) << 6) | (wave << 10) | ((uint32_t)(r >> 4) << 13)] =
                    __builtin_bit_cast(uint32_t, v[sub * 32 + r]);
        } else {
#pragma unroll
            for (int r = 0; r < 32; ++r) { // LB register r = (u5..u8, u13)
                const uint32_t q = r & 15, r4 = r >> 4;
                xbuf[lo | (((q & 1u) ^ l5) << 5) | (l5 << 6) | (wave << 7) | ((q >> 1) << 10) | (r4 << 13)] =
                    __builtin_bit_cast(uint32_t, v[sub * 32 + r]);
            }
        }
        __syncthreads();
        if (FORWARD) {
#pragma unroll
            for (int r = 0; r < 32; ++r) {
                const uint32_t q = r & 15, r4 = r >> 4;
                v[sub * 32 + r] = __builtin_bit_cast(
                    T, xbuf[lo | (((q & 1u) ^ l5) << 5) | (l5 << 6) | (wave << 7) | ((q >> 1) << 10) | (r4 << 13)]);
            }
        } else {
#pragma unroll
            for (int r = 0; r < 32; ++r)
                v[sub * 32 + r] = __builtin_bit_cast(
                    T, xbuf[lo | ((l5 ^ (uint32_t)(r & 1)) << 5) | ((uint32_t)(r & 15) << 6) | (wave << 10) | ((uint32_t)(r >> 4) << 13)]);
        }
    }
}

template <int MODE>
__global__ __launch_bounds__(kThreads, (MODE == SM_SERVER ? 2 : 4)) void k_strided(const StridedArgs a, const PtrTab tab)
{
    using TIN = typename std::conditional<(MODE == SM_ENC_FIRST || MODE == SM_MID_F32), float, int32_t>::type;
    __shared__ uint32_t lds[kLdsWords];
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const red = reinterpret_cast<float *>(lds + kXWords + kEpsWords + kLamWords);

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x, slot = blockIdx.y;
    const uint32_t cb = (uint32_t)kTileLog2 - a.hb;
    const bool need_x = cb < 9u;
    StridedGeom g;
    g.cb = cb;
    g.ls = a.ls;
    {
        const uint32_t sh = a.ls - cb;                    // column groups per outer block = 2^sh
        const uint64_t outer = (uint64_t)tile >> sh, cg = tile & ((1u << sh) - 1u);
        g.origin = (outer << (a.ls + a.hb)) + (cg << cb);
    }
    const uint64_t gb = g.origin >> a.logb;               // the tile lies inside one block

    // thread parts of the tile coordinate and of the element offset in both layouts
    const uint32_t uta = ua_thread(lane, wave), utb = ub_thread(lane, wave);
    const uint32_t ota = g.off(uta), otb = g.off(utb);
    // layout in which the transformed tile is held: LB if the exchange ran, else LA
    const uint32_t ut_out = need_x ? utb : uta, ot_out = need_x ? otb : ota;
    auto ureg_out = [&](int r) -> uint32_t { return need_x ? ub_reg(r) : ua_reg(r); };
    const uint32_t ebit = lane & 31u;

    TIN v[kV];

    if constexpr (MODE != SM_SERVER) {
        const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;
        const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, eps_party };
        if constexpr (MODE == SM_ENC_FIRST || MODE == SM_DEC_LAST) fill_eps(epsw, g, key_eps, t);

        // ---------------------------------------------------------------- load (LA)
        if constexpr (MODE == SM_ENC_FIRST) {
            const float *src = (a.use_tab ? tab.p[slot] : static_cast<const float *>(a.src) + slot * a.src_stride);
            const uint64_t room = a.len_in > g.origin ? a.len_in - g.origin : 0; // valid elements from the origin on
            src += g.origin;
#pragma unroll
            for (int r = 0; r < kV; ++r) {
                const uint32_t o = ota + g.off(ua_reg(r));
                v[r] = (o < room) ? src[o] : 0.f;
            }
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < kV; r += 4)
                acc += (v[r] * v[r] + v[r + 1] * v[r + 1]) + (v[r + 2] * v[r + 2] + v[r + 3] * v[r + 3]);
            acc = wave_sum(acc, 6);
            if (lane == 0) red[wave] = acc;
            __syncthreads(); // also publishes epsw
            if (t == 0) {
                float s = 0.f;
                for (int w = 0; w < 8; ++w) s += red[w];
                a.partials[(uint64_t)slot * gridDim.x + tile] = s;
            }
#pragma unroll
            for (int r = 0; r < kV; ++r) {
                const uint32_t w = epsw[(uta >> 5) + (ua_reg(r) >> 5)];
                v[r] = flip_if(v[r], (w >> ebit) & 1u);
            }
        } else {
            const TIN *src = static_cast<const TIN *>(a.src) + slot * a.src_stride + g.origin;
#pragma unroll
            for (int r = 0; r < kV; ++r) v[r] = src[ota + g.off(ua_reg(r))];
        }

        // ---------------------------------------------------------------- stages
        stages_a<TIN>(v, cb);
        if (need_x) {
            exchange<TIN, true>(v, xbuf, lane, wave);
            stages_b<TIN>(v, cb);
        } else if (MODE == SM_DEC_LAST) {
            __syncthreads(); // publishes epsw
        }

        // ---------------------------------------------------------------- store
        if constexpr (MODE == SM_DEC_LAST) {
            const float c = a.scales[slot * a.scales_stride + gb] * a.out_coef;
            float *dst = static_cast<float *>(a.dst) + g.origin;
            const uint64_t room = a.len_out > g.origin ? a.len_out - g.origin : 0;
#pragma unroll
            for (int r = 0; r < kV; ++r) {
                const uint32_t ur = ureg_out(r);
                const uint32_t o = ot_out + g.off(ur);
                const float val = flip_if(c * (float)v[r], (epsw[(ut_out >> 5) + (ur >> 5)] >> ebit) & 1u);
                if (o < room) {
                    if (a.store_mode == STORE_SET) dst[o] = val;
                    else if (a.store_mode == STORE_ACC) dst[o] += val;
                    else dst[o] -= a.delta * val;
                }
            }
        } else {
            TIN *dst = static_cast<TIN *>(a.dst) + slot * a.dst_stride + g.origin;
#pragma unroll
            for (int r = 0; r < kV; ++r) dst[ot_out + g.off(ureg_out(r))] = v[r];
        }
    } else {
        // ==================================================================== server
        float acc[kV];
#pragma unroll
        for (int r = 0; r < kV; ++r) acc[r] = 0.f;
        for (uint32_t m = 0; m < a.M; ++m) {
            const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, m };
            __syncthreads(); // previous iteration has finished reading epsw and xbuf
            fill_eps(epsw, g, key_eps, t);
            const int32_t *src = static_cast<const int32_t *>(a.src) + (uint64_t)m * a.src_stride + g.origin;
#pragma unroll
            for (int r = 0; r < kV; ++r) v[r] = src[ota + g.off(ua_reg(r))];
            stages_a<int32_t>(v, cb);
            if (need_x) {
                exchange<int32_t, true>(v, xbuf, lane, wave);
                stages_b<int32_t>(v, cb);
            } else {
                __syncthreads();
            }
            const float c = a.scales[(uint64_t)m * a.scales_stride + gb] * a.out_coef;
#pragma unroll
            for (int r = 0; r < kV; ++r)
                acc[r] += flip_if(c * (float)v[r], (epsw[(ut_out >> 5) + (ureg_out(r) >> 5)] >> ebit) & 1u);
        }
        if (a.gbar) {
            float *gq = a.gbar + g.origin;
#pragma unroll
            for (int r = 0; r < kV; ++r) gq[ot_out + g.off(ureg_out(r))] = acc[r];
        }
        // re-encode: eps^s flip, then the same stages in reverse layout order
        const RngKey key_s = { a.k0, a.k1, kDomainEps, a.round_lo, a.eps_party0 };
        __syncthreads();
        fill_eps(epsw, g, key_s, t);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < kV; ++r)
            acc[r] = flip_if(acc[r], (epsw[(ut_out >> 5) + (ureg_out(r) >> 5)] >> ebit) & 1u);
        if (need_x) {
            stages_b<float>(acc, cb);
            exchange<float, false>(acc, xbuf, lane, wave);
        }
        stages_a<float>(acc, cb);
        float *dst = static_cast<float *>(a.dst) + g.origin;
#pragma unroll
        for (int r = 0; r < kV; ++r) dst[ota + g.off(ua_reg(r))] = acc[r];
    }
}

} // namespace fo
