// Strided-tile kernel: up to ten Walsh-Hadamard stages on index bits above the contiguous tile
// (transform lengths above 2^15).  A tile is R = 2^hb rows by 2^(15-hb) consecutive columns, rows
// 2^ls coordinates apart; the stages act along the rows' axis only.
//
// Tile coordinate u = row << cb | col (cb = 15 - hb >= 5).  A thread holds 2^LV values as pairs of
// neighbouring columns (LV = 6: 512 threads x 64 values; LV = 5: 1024 threads x 32 values), so every global
// access moves a pair: 8 bytes per lane for fp32, 4 bytes per lane for the int16 intermediate that the decode
// side reads.  With NW = 9 - LV wave bits (see SL<LV>):
//   LA (loads):              reg0 = u0  lanes = (u1..u6)  waves = (u7..u6+NW)      regs 1.. = (u7+NW..u14)
//   LB (after the exchange): reg0 = u0  lanes = (u1..u6)  waves = (u7+NW..u6+2NW)  regs 1..NW = (u7..u6+NW)
// The exchange swaps the wave bits with register bits 1..NW through LDS (in two halves, one per pair member;
// the server pass does it in one whole-tile pass); lanes keep their bits, so LDS accesses are conflict free and
// stores are as coalesced as loads.  Row bits that fall on lane bits 4 and 5 (hb >= 9) are handled with
// v_permlane16_swap / v_permlane32_swap.
// Modes
//   SM_ENC_FIRST : fp32 gradient (zero padded), eps flip on load, tile sum of squares -> fp32 intermediate
//   SM_DEC_LAST  : integer intermediate -> lambda/sqrt(b) scaling, eps flip, store / SGD update (Def. 3.8)
//   SM_MID       : intermediate in, intermediate out (three-pass transforms)
//   SM_SERVER    : for every worker: int16 intermediate -> remaining inverse stages, scale, flip,
//                  accumulate the mean (eq. "server average"); then eps^s flip and the forward
//                  stages of the re-encode (Sec. 4, server-to-workers encoding) -> fp32 intermediate
//   SM_SHARED    : the same server step when all workers share one eps and one amplitude: the int32
//                  intermediate already holds the low stages of H^T sum_n q_n, so one tile is read, not M
#pragma once
#include "fo_contig.h"

namespace fo {

enum { SM_ENC_FIRST = 0, SM_DEC_LAST = 1, SM_MID_F32 = 2, SM_MID_I32 = 3, SM_SERVER = 4, SM_SHARED = 5 };

struct StridedArgs {
    const void *src;       // [slot][ntot] fp32 / int32 / int16 (ENC_FIRST: gradients, or pointer table)
    uint64_t src_stride;   // elements between slots
    void *dst;             // [slot][ntot] fp32 / int32; DEC_LAST: fp32 [len_out]
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
    const unsigned long long *round_dev; // optional: round counter read at run time
    float out_coef;        // value = lambda * out_coef * (transformed integer)
    float delta;
    // Padding of an intermediate that the neighbouring contiguous pass reads or writes tile by tile: row R (2^ls elements)
    // starts at R * (2^ls + pad) elements, which keeps rows that are a power of two apart off the same memory channels.
    uint32_t dst_pad;      // ENC_FIRST, SERVER, SHARED: fp32 destination
    uint32_t src_pad;      // DEC_LAST, SERVER with the int16 source
};

// Element offset of tile coordinate u from the tile origin.  Each bit of u has a fixed weight
// (column bits keep theirs, row bits move up to the row stride), so off(u1 | u2) = off(u1) + off(u2)
// for disjoint bit sets: a thread adds its own part once and a wave-uniform part per register pair.
struct StridedGeom {
    uint64_t origin; // coordinate of u = 0
    uint32_t cb, ls;
    __device__ __forceinline__ uint32_t off(uint32_t u) const
    {
        return ((u >> cb) << ls) + (u & ((1u << cb) - 1u));
    }
};

// Layout constants for V = 2^LV values per thread (as V/2 pairs) and 2^(15-LV) threads.
//   LA: reg0 = u0, lanes = (u1..u6), waves = (u7..u6+NW), register bits 1.. = (u7+NW..u14)
//   LB: reg0 = u0, lanes = (u1..u6), waves = (u7+NW..u6+2NW), register bits 1..NW = (u7..u6+NW),
//       register bits above NW unchanged
template <int LV>
struct SL {
    static constexpr int V = 1 << LV;       // values per thread
    static constexpr int P = V / 2;         // pairs per thread
    static constexpr int T = (int)kTile >> LV;
    static constexpr int NW = 9 - LV;       // wave bits: 3 for V = 64, 4 for V = 32
    static constexpr int NR = LV - 1;       // register bits other than the pair bit
    static_assert(NR >= NW, "the exchange needs as many register bits as wave bits");
    // thread part and (wave-uniform) pair part of a tile coordinate; p = register number >> 1
    static __device__ __forceinline__ uint32_t ta(uint32_t lane, uint32_t wave) { return (lane << 1) | (wave << 7); }
    static __device__ __forceinline__ constexpr uint32_t pa(int p) { return (uint32_t)p << (7 + NW); }
    static __device__ __forceinline__ uint32_t tb(uint32_t lane, uint32_t wave) { return (lane << 1) | (wave << (7 + NW)); }
    static __device__ __forceinline__ constexpr uint32_t pb(int p)
    {
        return ((uint32_t)(p & ((1 << NW) - 1)) << 7) | ((uint32_t)(p >> NW) << (7 + 2 * NW));
    }
};

// Load through a base pointer that is the same in every lane (held in scalar registers: the load takes the
// "scalar base + 32-bit lane offset" addressing form instead of 64-bit vector adds) plus a per-lane byte offset.
template <typename T>
__device__ __forceinline__ T ld_uniform(const void *uniform_base, uint32_t byte_off)
{
    typedef const __attribute__((address_space(1))) char *gptr;
    const uint64_t v = reinterpret_cast<uint64_t>(uniform_base);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    const gptr g = (gptr)(((uint64_t)hi << 32) | lo);
    return *(const __attribute__((address_space(1))) T *)(g + byte_off);
}

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
template <typename T>
__device__ __forceinline__ void st_uniform(void *uniform_base, uint32_t byte_off, T value)
{
    typedef __attribute__((address_space(1))) char *gptr;
    const uint64_t v = reinterpret_cast<uint64_t>(uniform_base);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    const gptr g = (gptr)(((uint64_t)hi << 32) | lo);
    *(__attribute__((address_space(1))) T *)(g + byte_off) = value;
}

// Access through a wave-uniform base pointer plus a 32-bit per-lane byte offset.
template <typename T>
__device__ __forceinline__ T ld_at(const void *uniform_base, uint32_t byte_off)
{
    return *reinterpret_cast<const T *>(static_cast<const char *>(uniform_base) + byte_off);
}
template <typename T>
__device__ __forceinline__ T &ref_at(void *uniform_base, uint32_t byte_off)
{
    return *reinterpret_cast<T *>(static_cast<char *>(uniform_base) + byte_off);
}

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

// One stage on lane bit 4 (partner = lane ^ 16): v_permlane16_swap trades the odd 16-lane rows of
// its first operand with the even rows of its second.
template <typename T, int V>
__device__ __forceinline__ void bfly_lane4(T (&v)[V])
{
#pragma unroll
    for (int k = 0; k < V / 2; ++k) {
        uint32_t a = __builtin_bit_cast(uint32_t, v[k]), b = __builtin_bit_cast(uint32_t, v[k + V / 2]);
        auto r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
        const T x = __builtin_bit_cast(T, (uint32_t)r[0]), y = __builtin_bit_cast(T, (uint32_t)r[1]);
        a = __builtin_bit_cast(uint32_t, (T)(x + y));
        b = __builtin_bit_cast(uint32_t, (T)(x - y));
        r = __builtin_amdgcn_permlane16_swap(a, b, false, false);
        v[k] = __builtin_bit_cast(T, (uint32_t)r[0]);
        v[k + V / 2] = __builtin_bit_cast(T, (uint32_t)r[1]);
    }
}

// stages on lane bits 4, 5 (u5, u6) and on the register bits of LA (register bit k <-> u bit 6 + NW + k)
template <typename T, int LV>
__device__ __forceinline__ void stages_a(T (&v)[1 << LV], uint32_t cb)
{
    constexpr int V = 1 << LV, B1 = 7 + SL<LV>::NW; // u bit of register bit 1
    if (cb <= 5u) bfly_lane4<T, V>(v);
    if (cb <= 6u) bfly_lane5<T, V>(v);
    if (cb <= (uint32_t)B1) bfly<T, 1, V>(v);
    if (cb <= (uint32_t)B1 + 1) bfly<T, 2, V>(v);
    if (cb <= (uint32_t)B1 + 2) bfly<T, 3, V>(v);
    if (cb <= (uint32_t)B1 + 3) bfly<T, 4, V>(v);
    if constexpr (LV > 5) {
        if (cb <= (uint32_t)B1 + 4) bfly<T, 5, V>(v);
    }
}
// stages on register bits 1..NW of LB (u7 ..)
template <typename T, int LV>
__device__ __forceinline__ void stages_b(T (&v)[1 << LV], uint32_t cb)
{
    constexpr int V = 1 << LV;
    if (cb <= 7u) bfly<T, 1, V>(v);
    if (cb <= 8u) bfly<T, 2, V>(v);
    if (cb <= 9u) bfly<T, 3, V>(v);
    if constexpr (SL<LV>::NW > 3) {
        if (cb <= 10u) bfly<T, 4, V>(v);
    }
}

// LA <-> LB through LDS: the wave index and register bits 1..NW trade places (the map is its own
// inverse).  Two halves, one per member of the pairs, so a lane moves 4 bytes per access and the
// lanes of a wave hit consecutive words.
// Word address: lane | wave-bits << 6 | register-bits-1..NW << (6 + NW) | higher register bits << (6 + 2 NW).
template <typename T, int LV>
__device__ __forceinline__ void exchange(T (&v)[1 << LV], uint32_t *xbuf, uint32_t lane, uint32_t wave)
{
    constexpr int P = SL<LV>::P, NW = SL<LV>::NW;
    uint32_t *const wp = xbuf + (lane | (wave << 6));
    uint32_t *const rp = xbuf + (lane | (wave << (6 + NW)));
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
        if (sub) __syncthreads();
#pragma unroll
        for (int p = 0; p < P; ++p)
            wp[((p & ((1 << NW) - 1)) << (6 + NW)) | ((p >> NW) << (6 + 2 * NW))] = __builtin_bit_cast(uint32_t, v[2 * p + sub]);
        __syncthreads();
#pragma unroll
        for (int p = 0; p < P; ++p)
            v[2 * p + sub] = __builtin_bit_cast(T, rp[((p & ((1 << NW) - 1)) << 6) | ((p >> NW) << (6 + 2 * NW))]);
    }
}

// The same exchange in one pass, both members of a pair in one 8-byte access: needs room for the whole
// tile (2^15 words), which a kernel that runs one workgroup per CU anyway can afford, and costs two
// barriers less per call.
template <typename T, int LV>
__device__ __forceinline__ void exchange_wide(T (&v)[1 << LV], uint32_t *xbuf, uint32_t lane, uint32_t wave)
{
    constexpr int P = SL<LV>::P, NW = SL<LV>::NW;
    uint2 *const wp = reinterpret_cast<uint2 *>(xbuf) + (lane | (wave << 6));
    const uint2 *const rp = reinterpret_cast<const uint2 *>(xbuf) + (lane | (wave << (6 + NW)));
#pragma unroll
    for (int p = 0; p < P; ++p)
        wp[((p & ((1 << NW) - 1)) << (6 + NW)) | ((p >> NW) << (6 + 2 * NW))] =
            make_uint2(__builtin_bit_cast(uint32_t, v[2 * p]), __builtin_bit_cast(uint32_t, v[2 * p + 1]));
    __syncthreads();
#pragma unroll
    for (int p = 0; p < P; ++p) {
        const uint2 d = rp[((p & ((1 << NW) - 1)) << 6) | ((p >> NW) << (6 + 2 * NW))];
        v[2 * p] = __builtin_bit_cast(T, d.x);
        v[2 * p + 1] = __builtin_bit_cast(T, d.y);
    }
}

// flip a pair by bits 2k, 2k+1 of an eps word already shifted right by 2k
__device__ __forceinline__ void flip_pair(float &x0, float &x1, uint32_t wshift)
{
    x0 = __uint_as_float(__float_as_uint(x0) ^ (wshift << 31));
    x1 = __uint_as_float(__float_as_uint(x1) ^ ((wshift << 30) & 0x80000000u));
}

// Tail of the server passes, on the mean of one tile held in layout LB (LA if no row bit lives in the wave index):
// optional copy of the mean, the tile's sum of squares for the measured-norm amplitude, eps^s flip, the forward
// stages of the re-encode in reverse layout order, store of the fp32 intermediate (Sec. 4, server-to-workers encoding).
// All threads of the workgroup call it; xbuf (kTile words if WIDE, else kXWords) and epsw (kEpsWords) are free on entry.
template <int LV, bool WIDE>
__device__ __forceinline__ void server_reencode(float (&acc)[1 << LV], const StridedArgs &a, const StridedGeom &g, uint32_t tile,
                                                uint32_t rk1, uint32_t rlo, uint32_t *xbuf, uint32_t *epsw, float *red, bool need_x)
{
    using L = SL<LV>;
    constexpr int kSV = L::V, kSP = L::P;
    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t cb = g.cb;
    const uint32_t uta = L::ta(lane, wave), utb = L::tb(lane, wave);
    const uint32_t ota = g.off(uta), otb = g.off(utb);
    const uint32_t ut_out = need_x ? utb : uta, ot_out = need_x ? otb : ota;
    auto upair_out = [&](int p) -> uint32_t { return need_x ? L::pb(p) : L::pa(p); };
    const uint32_t eshift = (lane & 15u) << 1;
    if (a.gbar) {
        float *gq = a.gbar + g.origin;
#pragma unroll
        for (int p = 0; p < kSP; ++p)
            ref_at<float2>(gq + g.off(upair_out(p)), ot_out * 4u) = make_float2(acc[2 * p], acc[2 * p + 1]);
    }
    // measured-norm server amplitude: this tile's sum of squares of the mean (the eps flip does not change it)
    if (a.partials) {
        float ss = 0.f;
#pragma unroll
        for (int r = 0; r < kSV; r += 4)
            ss += (acc[r] * acc[r] + acc[r + 1] * acc[r + 1]) + (acc[r + 2] * acc[r + 2] + acc[r + 3] * acc[r + 3]);
        ss = wave_sum(ss, 6);
        __syncthreads(); // red is free
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        if (t == 0) {
            float tot = 0.f;
            for (int w = 0; w < L::T / 64; ++w) tot += red[w];
            a.partials[tile] = tot;
        }
    }
    // re-encode: eps^s flip, then the same stages in reverse layout order
    const RngKey key_s = { a.k0, rk1, kDomainEps, rlo, a.eps_party0 };
    __syncthreads();
    fill_eps<L::T>(epsw, g, key_s, t);
    __syncthreads();
#pragma unroll
    for (int p = 0; p < kSP; ++p)
        flip_pair(acc[2 * p], acc[2 * p + 1], epsw[(ut_out >> 5) + (upair_out(p) >> 5)] >> eshift);
    if (need_x) {
        stages_b<float, LV>(acc, cb);
        if constexpr (WIDE) exchange_wide<float, LV>(acc, xbuf, lane, wave);
        else exchange<float, LV>(acc, xbuf, lane, wave);
    }
    stages_a<float, LV>(acc, cb);
    float *dst = static_cast<float *>(a.dst) + g.origin + (g.origin >> g.ls) * a.dst_pad;
    const uint32_t otd = ota + (uta >> cb) * a.dst_pad;
#pragma unroll
    for (int p = 0; p < kSP; ++p)
        ref_at<float2>(dst + g.off(L::pa(p)) + (L::pa(p) >> cb) * a.dst_pad, otd * 4u) = make_float2(acc[2 * p], acc[2 * p + 1]);
}

// HB = 0: the number of stages and the row stride are read from the arguments.  HB > 0: compiled
// for exactly HB stages with rows 2^15 apart (the pass next to the contiguous tile), which turns
// every per-register offset into a constant and removes the stage-selection branches.
// IN16: the integer input is the contiguous kernel's int16 intermediate.
// LV: log2 of the values per thread (6: 512 threads; 5: 1024 threads, used where two tiles' worth of
// registers per thread are needed and more waves hide latency better).
template <int MODE, int HB, bool IN16, int LV>
__global__ __launch_bounds__(SL<LV>::T, 4) void k_strided(const StridedArgs a, const PtrTab tab)
{
    using L = SL<LV>;
    constexpr int kSV = L::V, kSP = L::P;
    constexpr bool FIN = (MODE == SM_ENC_FIRST || MODE == SM_MID_F32); // fp32 input
    using TV = typename std::conditional<FIN, float, int32_t>::type;
    // the server pass holds so many registers that one workgroup fills a CU: it takes the whole-tile exchange
    constexpr bool WIDE = (MODE == SM_SERVER);
    constexpr uint32_t kXW = WIDE ? kTile : kXWords;
    __shared__ uint32_t lds[kXW + (WIDE ? 2u : 1u) * kEpsWords + kRedWords]; // the server pass alternates two eps tables
    uint32_t *const xbuf = lds;
    uint32_t *const epsw = lds + kXW;
    float *const red = reinterpret_cast<float *>(lds + kXW + (WIDE ? 2u : 1u) * kEpsWords);

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t slot = blockIdx.y;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    const uint32_t hb = HB ? (uint32_t)HB : a.hb;
    const uint32_t cb = (uint32_t)kTileLog2 - hb;
    // 64-byte row segments (int16 input, 32 columns): neighbouring column groups share 128-byte lines, so
    // they are given block indices that land on the same XCD (blocks are dealt round-robin over 8 XCDs)
    uint32_t tile = blockIdx.x;
    if (IN16 && cb == 5u) tile = (tile & ~15u) | ((tile & 7u) << 1) | ((tile >> 3) & 1u);
    const bool need_x = cb <= 6u + (uint32_t)L::NW; // some row bit lives in the wave index
    StridedGeom g;
    g.cb = cb;
    g.ls = HB ? (uint32_t)kTileLog2 : a.ls;
    {
        const uint32_t sh = g.ls - cb; // column groups per outer block = 2^sh
        const uint64_t outer = (uint64_t)tile >> sh, cg = tile & ((1u << sh) - 1u);
        g.origin = (outer << (g.ls + hb)) + (cg << cb);
    }
    const uint64_t gb = g.origin >> a.logb; // the tile lies inside one block

    // thread parts of the tile coordinate and of the element offset in both layouts
    const uint32_t uta = L::ta(lane, wave), utb = L::tb(lane, wave);
    const uint32_t ota = g.off(uta), otb = g.off(utb);
    // layout in which the transformed tile is held: LB if the exchange ran, else LA
    const uint32_t ut_out = need_x ? utb : uta, ot_out = need_x ? otb : ota;
    auto upair_out = [&](int p) -> uint32_t { return need_x ? L::pb(p) : L::pa(p); };
    const uint32_t eshift = (lane & 15u) << 1; // bit of column u0 = 0 inside its eps word

    // ---- input of one tile (layout LA) as 32 pairs
    auto load_int = [&](int32_t (&v)[kSV], const void *src_base) {
        const uint32_t spad = IN16 ? a.src_pad : 0u;
        const uint32_t otp = ota + (uta >> cb) * spad;
#pragma unroll
        for (int p = 0; p < kSP; ++p) {
            const uint32_t ro = g.off(L::pa(p)) + (L::pa(p) >> cb) * spad; // wave-uniform
            if constexpr (IN16) {
                const uint32_t d = ld_at<uint32_t>(static_cast<const int16_t *>(src_base) + ro, otp * 2u);
                v[2 * p] = (int32_t)(int16_t)(d & 0xFFFFu);
                v[2 * p + 1] = (int32_t)d >> 16;
            } else {
                const int2 d = ld_at<int2>(static_cast<const int32_t *>(src_base) + ro, ota * 4u);
                v[2 * p] = d.x;
                v[2 * p + 1] = d.y;
            }
        }
    };

    if constexpr (MODE != SM_SERVER && MODE != SM_SHARED) {
        TV v[kSV];
        const uint32_t eps_party = (a.eps_party0 >= 0xFFFFFFFEu) ? a.eps_party0 : a.eps_party0 + slot;
        const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, eps_party };
        if constexpr (MODE == SM_ENC_FIRST || MODE == SM_DEC_LAST) fill_eps<L::T>(epsw, g, key_eps, t);

        // ---------------------------------------------------------------- load (LA)
        if constexpr (MODE == SM_ENC_FIRST) {
            const float *src = (a.use_tab ? tab.p[slot] : static_cast<const float *>(a.src) + slot * a.src_stride);
            const uint64_t room = a.len_in > g.origin ? a.len_in - g.origin : 0; // valid elements from the origin on
            src += g.origin;
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                const uint32_t ro = g.off(L::pa(p)); // wave-uniform
                const uint64_t e = (uint64_t)ro + ota;
                float2 d = make_float2(0.f, 0.f);
                if (e + 1 < room) {
                    const f32x2 q = ld_uniform<f32x2>(src + ro, ota * 4u);
                    d = make_float2(q.x, q.y);
                } else if (e < room) {
                    d.x = ld_uniform<float>(src + ro, ota * 4u);
                }
                v[2 * p] = d.x;
                v[2 * p + 1] = d.y;
            }
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < kSV; r += 4)
                acc += (v[r] * v[r] + v[r + 1] * v[r + 1]) + (v[r + 2] * v[r + 2] + v[r + 3] * v[r + 3]);
            acc = wave_sum(acc, 6);
            if (lane == 0) red[wave] = acc;
            __syncthreads(); // also publishes epsw
            if (t == 0) {
                float s = 0.f;
                for (int w = 0; w < L::T / 64; ++w) s += red[w];
                a.partials[(uint64_t)slot * gridDim.x + tile] = s;
            }
#pragma unroll
            for (int p = 0; p < kSP; ++p)
                flip_pair(v[2 * p], v[2 * p + 1], epsw[(uta >> 5) + (L::pa(p) >> 5)] >> eshift);
        } else if constexpr (MODE == SM_MID_F32) {
            const float *src = static_cast<const float *>(a.src) + slot * a.src_stride + g.origin;
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                const float2 d = ld_at<float2>(src + g.off(L::pa(p)), ota * 4u);
                v[2 * p] = d.x;
                v[2 * p + 1] = d.y;
            }
        } else {
            const char *src = static_cast<const char *>(a.src) + (slot * a.src_stride + g.origin + (IN16 ? (g.origin >> g.ls) * a.src_pad : 0u)) * (IN16 ? 2u : 4u);
            load_int(v, src);
        }

        // ---------------------------------------------------------------- stages
        stages_a<TV, LV>(v, cb);
        if (need_x) {
            exchange<TV, LV>(v, xbuf, lane, wave);
            stages_b<TV, LV>(v, cb);
        } else if (MODE == SM_DEC_LAST) {
            __syncthreads(); // publishes epsw
        }

        // ---------------------------------------------------------------- store
        if constexpr (MODE == SM_DEC_LAST) {
            const float c = a.scales[slot * a.scales_stride + gb] * a.out_coef;
            float *dst = static_cast<float *>(a.dst) + g.origin;
            const uint64_t room = a.len_out > g.origin ? a.len_out - g.origin : 0;
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                const uint32_t up = upair_out(p);
                const uint32_t ro = g.off(up); // wave-uniform
                float y0 = c * (float)v[2 * p], y1 = c * (float)v[2 * p + 1];
                flip_pair(y0, y1, epsw[(ut_out >> 5) + (up >> 5)] >> eshift);
                const uint64_t e = (uint64_t)ro + ot_out;
                if (e + 1 < room) {
                    float2 &q = ref_at<float2>(dst + ro, ot_out * 4u);
                    if (a.store_mode == STORE_SET) q = make_float2(y0, y1);
                    else if (a.store_mode == STORE_ACC) q = make_float2(q.x + y0, q.y + y1);
                    else q = make_float2(q.x - a.delta * y0, q.y - a.delta * y1);
                } else if (e < room) {
                    float &q = ref_at<float>(dst + ro, ot_out * 4u);
                    if (a.store_mode == STORE_SET) q = y0;
                    else if (a.store_mode == STORE_ACC) q += y0;
                    else q -= a.delta * y0;
                }
            }
        } else {
            const uint32_t pad = (MODE == SM_ENC_FIRST) ? a.dst_pad : 0u;
            TV *dst = static_cast<TV *>(a.dst) + slot * a.dst_stride + g.origin + (g.origin >> g.ls) * pad;
            const uint32_t ot_pad = ot_out + (ut_out >> cb) * pad;
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                using T2 = typename std::conditional<FIN, f32x2, i32x2>::type;
                T2 d;
                d.x = v[2 * p];
                d.y = v[2 * p + 1];
                const uint32_t up = upair_out(p);
                st_uniform<T2>(dst + g.off(up) + (up >> cb) * pad, ot_pad * 4u, d);
            }
        }
    } else {
        // ==================================================================== server
        float acc[kSV];
        if constexpr (MODE == SM_SHARED) {
            // one tile: remaining inverse stages of H^T (sum of the workers' sign vectors), amplitude / M, shared eps
            static_assert(!IN16, "the summed sign vectors need an int32 intermediate");
            int32_t v[kSV];
            const RngKey key_w = { a.k0, rk1, kDomainEps, rlo, 0xFFFFFFFEu };
            fill_eps<L::T>(epsw, g, key_w, t);
            load_int(v, static_cast<const char *>(a.src) + g.origin * 4u);
            stages_a<int32_t, LV>(v, cb);
            if (need_x) {
                exchange<int32_t, LV>(v, xbuf, lane, wave);
                stages_b<int32_t, LV>(v, cb);
            } else {
                __syncthreads();
            }
            const float c = a.scales[gb] * a.out_coef;
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                acc[2 * p] = c * (float)v[2 * p];
                acc[2 * p + 1] = c * (float)v[2 * p + 1];
                flip_pair(acc[2 * p], acc[2 * p + 1], epsw[(ut_out >> 5) + (upair_out(p) >> 5)] >> eshift);
            }
        } else {
#pragma unroll
        for (int r = 0; r < kSV; ++r) acc[r] = 0.f;
        if constexpr (!IN16) {
            // int32 intermediate (three-pass transforms, blocks above 2^25): the values outgrow fp32's 24 bits, so the
            // remaining stages stay in integers, as in the decoder, and only the result is converted; no prefetch.
            for (uint32_t m = 0; m < a.M; ++m) {
                int32_t v[kSV];
                load_int(v, static_cast<const char *>(a.src) + ((uint64_t)m * a.src_stride + g.origin) * 4u);
                const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, m };
                uint32_t *const epsm = epsw + (m & 1u) * kEpsWords; // two tables in turn, as below
                fill_eps<L::T>(epsm, g, key_eps, t);
                stages_a<int32_t, LV>(v, cb);
                if (need_x) {
                    __syncthreads(); // the previous worker's exchange buffer is no longer read
                    exchange_wide<int32_t, LV>(v, xbuf, lane, wave);
                    stages_b<int32_t, LV>(v, cb);
                } else {
                    __syncthreads(); // publishes the eps table
                }
                const uint32_t cbits = __float_as_uint(a.scales[(uint64_t)m * a.scales_stride + gb] * a.out_coef);
#pragma unroll
                for (int p = 0; p < kSP; ++p) {
                    const uint32_t w = epsm[(ut_out >> 5) + (upair_out(p) >> 5)];
                    acc[2 * p] = fmaf((float)v[2 * p], __uint_as_float(((w >> eshift) << 31) + cbits), acc[2 * p]);
                    acc[2 * p + 1] = fmaf((float)v[2 * p + 1], __uint_as_float(((w >> (eshift + 1u)) << 31) + cbits), acc[2 * p + 1]);
                }
            }
        } else {
        uint32_t raw[kSP]; // packed tile of the next worker, in flight while the current one is transformed
        const uint32_t otp = ota + (uta >> cb) * a.src_pad;
        auto request = [&](uint32_t m) {
            const int16_t *src = static_cast<const int16_t *>(a.src) + (uint64_t)m * a.src_stride + g.origin + (g.origin >> g.ls) * a.src_pad;
#pragma unroll
            for (int p = 0; p < kSP; ++p) raw[p] = ld_uniform<uint32_t>(src + g.off(L::pa(p)) + (L::pa(p) >> cb) * a.src_pad, otp * 2u);
        };
        // finish worker m, whose packed tile is in `raw`; with PREFETCH the registers of `raw` are refilled
        // with worker m + 1 as soon as they have been unpacked
        auto process = [&](uint32_t m, auto prefetch) {
            constexpr bool PREFETCH = decltype(prefetch)::value;
            // fp32 butterflies: every value is an integer below 2^24 in magnitude, so each sum is exact
            float buf[kSV];
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                buf[2 * p] = (float)(int16_t)(raw[p] & 0xFFFFu);
                buf[2 * p + 1] = (float)((int32_t)raw[p] >> 16);
            }
            if constexpr (PREFETCH) request(m + 1);
            const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, m };
            // Two eps tables in turn: worker m's table is written while slow waves may still read worker m-1's,
            // and it is read after this iteration's barrier, which every wave reaches only when done with m-1.
            uint32_t *const epsm = epsw + (m & 1u) * kEpsWords;
            fill_eps<L::T>(epsm, g, key_eps, t);
            stages_a<float, LV>(buf, cb);
            if (need_x) {
                __syncthreads(); // the previous worker's exchange buffer is no longer read
                exchange_wide<float, LV>(buf, xbuf, lane, wave);
                stages_b<float, LV>(buf, cb);
            } else {
                __syncthreads(); // publishes the eps table
            }
            // acc += (+-c) * value: the eps bit is added into the coefficient's sign bit (a flip, whatever the sign was)
            const uint32_t cbits = __float_as_uint(a.scales[(uint64_t)m * a.scales_stride + gb] * a.out_coef);
#pragma unroll
            for (int p = 0; p < kSP; ++p) {
                const uint32_t w = epsm[(ut_out >> 5) + (upair_out(p) >> 5)];
                acc[2 * p] = fmaf(buf[2 * p], __uint_as_float(((w >> eshift) << 31) + cbits), acc[2 * p]);
                acc[2 * p + 1] = fmaf(buf[2 * p + 1], __uint_as_float(((w >> (eshift + 1u)) << 31) + cbits), acc[2 * p + 1]);
            }
        };
        request(0);
        for (uint32_t m = 0; m + 1 < a.M; ++m) {
            // generic geometry: keep the per-register row offsets (functions of ls) from being hoisted out of
            // this loop and held in scalar registers for its whole duration
            if constexpr (HB == 0) asm volatile("" : "+s"(g.ls));
            process(m, std::true_type{});
        }
        process(a.M - 1, std::false_type{});
        }
        }
        server_reencode<LV, WIDE>(acc, a, g, tile, rk1, rlo, xbuf, epsw, red, need_x);
    }
}

} // namespace fo
