// Strided-tile kernel: up to ten Walsh-Hadamard stages on index bits above the contiguous tile
// (transform lengths above 2^15).  A tile is R = 2^hb rows by 2^(15-hb) consecutive columns, rows
// 2^ls coordinates apart; the stages act along the rows' axis only.  Global accesses are one
// dword per lane; a wave touches 64 consecutive columns (256 B), or 2 x 32 when hb = 10.
//
// Tile coordinate u = row << cb | col (cb = 15 - hb).  With V = 2^LV values per thread and
// NW = 9 - LV wave bits (V = 64: 512 threads; V = 32: 1024 threads):
//   LA (loads):              lanes = (u0..u5)  waves = (u6..u5+NW)        regs = (u6+NW..u14)
//   LB (after the exchange): lanes = (u0..u5)  waves = (u6+NW..u5+2NW)    regs = (u6..u5+NW, u6+2NW..u14)
// The exchange swaps the wave bits with the low NW register bits through LDS; lanes keep their
// bits, so LDS accesses are conflict free and global stores stay as coalesced as the loads.  A row
// bit that falls on lane bit 5 (hb = 10) is handled with v_permlane32_swap.
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

// Access through a wave-uniform base pointer plus a 32-bit per-lane byte offset: this is the
// address form that needs one offset register per thread instead of a 64-bit address per access.
template <typename T>
__device__ __forceinline__ T ld_at(const T *uniform_base, uint32_t byte_off)
{
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(uniform_base) + byte_off);
}
template <typename T>
__device__ __forceinline__ T &ref_at(T *uniform_base, uint32_t byte_off)
{
    return *reinterpret_cast<T *>(reinterpret_cast<char *>(uniform_base) + byte_off);
}

template <int LV>
struct SLayout {
    static constexpr int V = 1 << LV;
    static constexpr int T = (int)kTile >> LV;
    static constexpr int NW = 9 - LV;                 // wave bits
    static constexpr int NS = LV - NW;                // register bits the exchange leaves alone
    static_assert(NS >= 1, "the exchange is split in two halves on a spectator register bit");
    // thread part and (wave-uniform) register part of a tile coordinate in the two layouts
    static __device__ __forceinline__ uint32_t ta(uint32_t lane, uint32_t wave) { return lane | (wave << 6); }
    static __device__ __forceinline__ constexpr uint32_t ra(int r) { return (uint32_t)r << (6 + NW); }
    static __device__ __forceinline__ uint32_t tb(uint32_t lane, uint32_t wave) { return lane | (wave << (6 + NW)); }
    static __device__ __forceinline__ constexpr uint32_t rb(int r)
    {
        return ((uint32_t)(r & ((1 << NW) - 1)) << 6) | ((uint32_t)(r >> NW) << (6 + 2 * NW));
    }
};

// eps words of the tile, one 32-bit word per group of 32 consecutive columns (u >> 5)
template <int T>
__device__ __forceinline__ void fill_eps(uint32_t *epsw, const StridedGeom &g, const RngKey &key, uint32_t t)
{
#pragma unroll
    for (int h = 0; h < 1024 / T; ++h) {
        const uint32_t grp = t + h * T;
        const uint64_t i = g.origin + g.off(grp << 5);
        uint32_t w[4];
        philox((uint32_t)(i >> 7), key, w);
        const uint32_t sel = (uint32_t)(i >> 5) & 3u;
        epsw[grp] = sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
    }
}

// stages on the register bits of LA (register bit k <-> u bit 6 + NW + k) and on lane bit 5
template <typename T, int LV>
__device__ __forceinline__ void stages_a(T (&v)[1 << LV], uint32_t cb)
{
    constexpr int B0 = 6 + SLayout<LV>::NW, V = 1 << LV;
    if (cb <= 5u) bfly_lane5<T, V>(v);
    if (cb <= (uint32_t)B0) bfly<T, 0, V>(v);
    if (cb <= (uint32_t)B0 + 1) bfly<T, 1, V>(v);
    if (cb <= (uint32_t)B0 + 2) bfly<T, 2, V>(v);
    if (cb <= (uint32_t)B0 + 3) bfly<T, 3, V>(v);
    if constexpr (LV > 4) {
        if (cb <= (uint32_t)B0 + 4) bfly<T, 4, V>(v);
    }
    if constexpr (LV > 5) {
        if (cb <= (uint32_t)B0 + 5) bfly<T, 5, V>(v);
    }
}
// stages on the low NW register bits of LB (register bit k <-> u bit 6 + k)
template <typename T, int LV>
__device__ __forceinline__ void stages_b(T (&v)[1 << LV], uint32_t cb)
{
    constexpr int NW = SLayout<LV>::NW, V = 1 << LV;
    if (cb <= 6u) bfly<T, 0, V>(v);
    if (cb <= 7u) bfly<T, 1, V>(v);
    if (cb <= 8u) bfly<T, 2, V>(v);
    if constexpr (NW > 3) {
        if (cb <= 9u) bfly<T, 3, V>(v);
    }
}

// LA <-> LB through LDS in two halves split on the top register bit (a spectator): the wave index
// and the low NW register bits trade places (the map is its own inverse).
// Word address: lane | wave-bits << 6 | low-register-bits << (6 + NW) | other spectators << (6 + 2 NW).
template <typename T, int LV>
__device__ __forceinline__ void exchange(T (&v)[1 << LV], uint32_t *xbuf, uint32_t lane, uint32_t wave)
{
    constexpr int V = 1 << LV, NW = SLayout<LV>::NW, H = V / 2;
    const uint32_t wofs = lane | (wave << 6), rofs = lane | (wave << (6 + NW));
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
        if (sub) __syncthreads();
#pragma unroll
        for (int r = 0; r < H; ++r)
            xbuf[wofs + ((r & ((1 << NW) - 1)) << (6 + NW)) + ((r >> NW) << (6 + 2 * NW))] =
                __builtin_bit_cast(uint32_t, v[sub * H + r]);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < H; ++r)
            v[sub * H + r] =
                __builtin_bit_cast(T, xbuf[rofs + ((r & ((1 << NW) - 1)) << 6) + ((r >> NW) << (6 + 2 * NW))]);
    }
}

// HB = 0: the number of stages and the row stride are read from the arguments.  HB > 0: compiled
// for exactly HB stages with rows 2^15 apart (the pass next to the contiguous tile), which turns
// every per-register offset into a constant and removes the stage-selection branches.
template <int MODE, int LV, int HB>
__global__ __launch_bounds__(SLayout<LV>::T, (MODE == SM_SERVER ? 2 : 4)) void k_strided(const StridedArgs a, const PtrTab tab)
{
    using L = SLayout<LV>;
    constexpr int V = L::V, T = L::T;
    using TIN = typename std::conditional<(MODE == SM_ENC_FIRST || MODE == SM_MID_F32), float, int32_t>::type;
    __shared__ uint32_t lds[kLdsWords];
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXWords;
    float *const red = reinterpret_cast<float *>(lds + kXWords + kEpsWords + kLamWords);

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t tile = blockIdx.x, slot = blockIdx.y;
    const uint32_t hb = HB ? (uint32_t)HB : a.hb;
    const uint32_t cb = (uint32_t)kTileLog2 - hb;
    const bool need_x = cb < 6u + (uint32_t)L::NW;      // some row bit lives in the wave index
    StridedGeom g;
    g.cb = cb;
    g.ls = HB ? (uint32_t)kTileLog2 : a.ls;
    {
        const uint32_t sh = g.ls - cb;                    // column groups per outer block = 2^sh
        const uint64_t outer = (uint64_t)tile >> sh, cg = tile & ((1u << sh) - 1u);
        g.origin = (outer << (g.ls + hb)) + (cg << cb);
    }
    const uint64_t gb = g.origin >> a.logb;               // the tile lies inside one block

    // thread parts of the tile coordinate and of the element offset in both layouts
    const uint32_t uta = L::ta(lane, wave), utb = L::tb(lane, wave);
    const uint32_t ota = g.off(uta), otb = g.off(utb);
    // layout in which the transformed tile is held: LB if the exchange ran, else LA
    const uint32_t ut_out = need_x ? utb : uta, ot_out = need_x ? otb : ota;
    auto ureg_out = [&](int r) -> uint32_t { return need_x ? L::rb(r) : L::ra(r); };
    const uint32_t ebit = lane & 31u;
    const uint32_t oba = ota * 4u, ob_out = ot_out * 4u; // per-thread byte offsets (tiles span < 2^32 bytes)

    if constexpr (MODE != SM_SERVER) {
        TIN v[V];
        const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;
        const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, eps_party };
        if constexpr (MODE == SM_ENC_FIRST || MODE == SM_DEC_LAST) fill_eps<T>(epsw, g, key_eps, t);

        // ---------------------------------------------------------------- load (LA)
        if constexpr (MODE == SM_ENC_FIRST) {
            const float *src = (a.use_tab ? tab.p[slot] : static_cast<const float *>(a.src) + slot * a.src_stride);
            const uint64_t room = a.len_in > g.origin ? a.len_in - g.origin : 0; // valid elements from the origin on
            src += g.origin;
#pragma unroll
            for (int r = 0; r < V; ++r) {
                const uint32_t ro = g.off(L::ra(r));             // wave-uniform part
                v[r] = ((uint64_t)ro + ota < room) ? ld_at(src + ro, oba) : 0.f;
            }
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < V; r += 4)
                acc += (v[r] * v[r] + v[r + 1] * v[r + 1]) + (v[r + 2] * v[r + 2] + v[r + 3] * v[r + 3]);
            acc = wave_sum(acc, 6);
            if (lane == 0) red[wave] = acc;
            __syncthreads(); // also publishes epsw
            if (t == 0) {
                float s = 0.f;
                for (int w = 0; w < T / 64; ++w) s += red[w];
                a.partials[(uint64_t)slot * gridDim.x + tile] = s;
            }
#pragma unroll
            for (int r = 0; r < V; ++r) {
                const uint32_t w = epsw[(uta >> 5) + (L::ra(r) >> 5)];
                v[r] = flip_if(v[r], (w >> ebit) & 1u);
            }
        } else {
            const TIN *src = static_cast<const TIN *>(a.src) + slot * a.src_stride + g.origin;
#pragma unroll
            for (int r = 0; r < V; ++r) v[r] = ld_at(src + g.off(L::ra(r)), oba);
        }

        // ---------------------------------------------------------------- stages
        stages_a<TIN, LV>(v, cb);
        if (need_x) {
            exchange<TIN, LV>(v, xbuf, lane, wave);
            stages_b<TIN, LV>(v, cb);
        } else if (MODE == SM_DEC_LAST) {
            __syncthreads(); // publishes epsw
        }

        // ---------------------------------------------------------------- store
        if constexpr (MODE == SM_DEC_LAST) {
            const float c = a.scales[slot * a.scales_stride + gb] * a.out_coef;
            float *dst = static_cast<float *>(a.dst) + g.origin;
            const uint64_t room = a.len_out > g.origin ? a.len_out - g.origin : 0;
#pragma unroll
            for (int r = 0; r < V; ++r) {
                const uint32_t ur = ureg_out(r);
                const uint32_t ro = g.off(ur);                   // wave-uniform part
                const float val = flip_if(c * (float)v[r], (epsw[(ut_out >> 5) + (ur >> 5)] >> ebit) & 1u);
                if ((uint64_t)ro + ot_out < room) {
                    float &q = ref_at(dst + ro, ob_out);
                    if (a.store_mode == STORE_SET) q = val;
                    else if (a.store_mode == STORE_ACC) q += val;
                    else q -= a.delta * val;
                }
            }
        } else {
            TIN *dst = static_cast<TIN *>(a.dst) + slot * a.dst_stride + g.origin;
#pragma unroll
            for (int r = 0; r < V; ++r) ref_at(dst + g.off(ureg_out(r)), ob_out) = v[r];
        }
    } else {
        // ==================================================================== server
        float acc[V];
        int32_t bufa[V], bufb[V]; // ping-pong: one tile is transformed while the next one travels
#pragma unroll
        for (int r = 0; r < V; ++r) acc[r] = 0.f;

        // request registers [r0, r1) of worker m's tile
        auto request = [&](int32_t (&buf)[V], uint32_t m, auto r0, auto r1) {
            const int32_t *src = static_cast<const int32_t *>(a.src) + (uint64_t)m * a.src_stride + g.origin;
#pragma unroll
            for (int r = decltype(r0)::value; r < decltype(r1)::value; ++r) buf[r] = ld_at(src + g.off(L::ra(r)), oba);
        };
        using I0 = std::integral_constant<int, 0>;
        using IH = std::integral_constant<int, V / 2>;
        using IV = std::integral_constant<int, V>;
        // finish worker m (tile in `buf`) while worker m + 1 is requested into `nbuf` in two batches, so
        // that the wait for `buf` never has more than V/2 younger loads in flight behind it
        auto process = [&](int32_t (&buf)[V], int32_t (&nbuf)[V], uint32_t m) {
            const bool more = m + 1 < a.M;
            if (more) request(nbuf, m + 1, I0{}, IH{});
            const RngKey key_eps = { a.k0, a.k1, kDomainEps, a.round_lo, m };
            __syncthreads(); // the previous worker's eps words and exchange buffer are no longer read
            fill_eps<T>(epsw, g, key_eps, t);
            stages_a<int32_t, LV>(buf, cb);
            if (more) request(nbuf, m + 1, IH{}, IV{});
            if (need_x) {
                exchange<int32_t, LV>(buf, xbuf, lane, wave);
                stages_b<int32_t, LV>(buf, cb);
            } else {
                __syncthreads();
            }
            const float c = a.scales[(uint64_t)m * a.scales_stride + gb] * a.out_coef;
#pragma unroll
            for (int r = 0; r < V; ++r)
                acc[r] += flip_if(c * (float)buf[r], (epsw[(ut_out >> 5) + (ureg_out(r) >> 5)] >> ebit) & 1u);
        };
        request(bufa, 0, I0{}, IV{});
        for (uint32_t m = 0; m < a.M; m += 2) {
            // keep the per-register row offsets (functions of ls) from being hoisted out of this loop
            // and held in scalar registers for its whole duration
            if constexpr (HB == 0) asm volatile("" : "+s"(g.ls));
            process(bufa, bufb, m);
            if (m + 1 < a.M) process(bufb, bufa, m + 1);
        }
        if (a.gbar) {
            float *gq = a.gbar + g.origin;
#pragma unroll
            for (int r = 0; r < V; ++r) ref_at(gq + g.off(ureg_out(r)), ob_out) = acc[r];
        }
        // re-encode: eps^s flip, then the same stages in reverse layout order
        const RngKey key_s = { a.k0, a.k1, kDomainEps, a.round_lo, a.eps_party0 };
        __syncthreads();
        fill_eps<T>(epsw, g, key_s, t);
        __syncthreads();
#pragma unroll
        for (int r = 0; r < V; ++r)
            acc[r] = flip_if(acc[r], (epsw[(ut_out >> 5) + (ureg_out(r) >> 5)] >> ebit) & 1u);
        if (need_x) {
            stages_b<float, LV>(acc, cb);
            exchange<float, LV>(acc, xbuf, lane, wave);
        }
        stages_a<float, LV>(acc, cb);
        float *dst = static_cast<float *>(a.dst) + g.origin;
#pragma unroll
        for (int r = 0; r < V; ++r) ref_at(dst + g.off(L::ra(r)), oba) = acc[r];
    }
}

} // namespace fo
