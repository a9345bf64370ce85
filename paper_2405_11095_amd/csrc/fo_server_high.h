// Server pass over the ten index bits above the contiguous tile (transform blocks of 2^25 coordinates) with the
// inverse stages on the matrix cores: for every worker, int16 intermediate -> remaining ten inverse stages,
// amplitude, eps flip, accumulate the mean (eq. "server average"); then the tail shared with the vector-unit
// kernel: eps^s flip and the forward stages of the re-encode (Sec. 4, server-to-workers encoding).
//
// A tile is 1024 rows (2^15 coordinates apart) by 32 consecutive columns; the stages act along the rows, so a
// column is one 1024-point transform, H_1024 = H_32 (x) H_32 with row = 32 rA + rB.  As in the decode-side tile
// kernels the data enter v_mfma_f32_32x32x16_f16 as the A operand (lane = a row index that is not being
// transformed, k = the one that is) and each product leaves the transformed index on the lanes and the old
// rows in the registers, so the second product contracts over the registers of the first with no data movement.
//
// The inputs are integers up to 2^14 in magnitude, more than fp16's eleven bits hold, so every stage takes its
// input as two fp16 pieces and runs two products:
//   stage A (rA -> tA): x = 128 (x >> 7) + (x & 127).  Both pieces are made in the integer domain, two per
//       instruction, as fp16 bit patterns whose exponent is chosen so that the significand counts in the wanted unit:
//       0x6400 + 128 + (x >> 7) is the number 1152 + (x >> 7), 0x4800 + (x & 127) is 8 + (x & 127) / 128.
//       Both go against H_32 / 4, so the product is the transform times 2^-9 (a power of two: still exact); the
//       biases add (1152 * 128 + 1024) * 32 / 512 to the outputs tA = 0 and nothing elsewhere (every other column
//       of H_32 sums to zero), and the accumulator of the product starts from minus that.
//   stage B (rB -> tB): the stage-A result is at most 2^10 with twenty significant bits: v_cvt_pkrtz keeps the
//       top eleven (first piece), the remainder, exact in fp32, has at most ten (second piece).  Both go against
//       the same H_32 / 4 (one constant operand for the whole kernel); the factor 2^11 is folded into the
//       amplitude.
// Every product and sum is an integer multiple of its unit below 2^24 units, so the result equals the
// vector-unit kernel's bit for bit.
//
// 1024 threads.  Global loads are the coalesced ones of the vector-unit kernel (16 lanes cover the 64 bytes of a
// row, one dword = a pair of columns); they are written to LDS as [column pair][rB][rA] and wave w reads column
// pair w from there in the operand's register order with 16-byte accesses.  The staging buffer and the eps
// table are doubled, which leaves one barrier per worker.
#pragma once
#include "fo_strided.h"
#include "fo_mfma.h"

namespace fo {

constexpr uint32_t kShRowWords = 36u;                     // the 32 rA of one (column pair, rB), padded to 36 words
constexpr uint32_t kShPairWords = 32u * kShRowWords + 4u; // one column pair; + 4 spreads the pairs over the banks
constexpr uint32_t kShStageWords = 16u * kShPairWords;    // one worker's tile
constexpr uint32_t kShTransPitch = 17u;                   // 8-byte units per row of the final transposition (16 pairs + 1)
constexpr uint32_t kShLdsWords = 2u * kShStageWords + 2u * 1024u + kRedWords + 32u; // + the two bias vectors
static_assert(1024u * kShTransPitch * 2u <= 2u * kShStageWords, "the transposition reuses the staging buffers");
static_assert(kTile <= 2u * kShStageWords, "the re-encode's exchange reuses the staging buffers");
static_assert(kShLdsWords * 4u <= 160u * 1024u, "LDS of a compute unit");

typedef short sh_s16x2 __attribute__((ext_vector_type(2)));
typedef unsigned short sh_u16x2 __attribute__((ext_vector_type(2)));

static __global__ __launch_bounds__(1024) void k_server_mfma(const StridedArgs a)
{
    constexpr int LV = 5;
    using L = SL<LV>;
    __shared__ __attribute__((aligned(16))) uint32_t lds[kShLdsWords];
    uint32_t *const epsw = lds + 2u * kShStageWords;
    float *const red = reinterpret_cast<float *>(lds + 2u * kShStageWords + 2u * 1024u);
    float *const bias_tab = reinterpret_cast<float *>(lds + 2u * kShStageWords + 2u * 1024u + kRedWords);

    const uint32_t t = threadIdx.x, lane = t & 63u, wave = t >> 6;
    const uint32_t col = lane & 31u, h = lane >> 5;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    // neighbouring column groups share 128-byte lines: give them block indices that land on the same XCD
    uint32_t tile = blockIdx.x;
    tile = (tile & ~15u) | ((tile & 7u) << 1) | ((tile >> 3) & 1u);
    StridedGeom g;
    g.cb = 5u;
    g.ls = (uint32_t)kTileLog2;
    g.origin = ((uint64_t)(tile >> 10) << 25) + ((uint64_t)(tile & 1023u) << 5);
    const uint64_t gb = g.origin >> a.logb;

    // constant operand of all products: H_32 / 4 in the k order of the operand registers
    mf_v8h bh[2];
#pragma unroll
    for (int mm = 0; mm < 2; ++mm)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const uint32_t k = 8u * (2u * mm + (e >> 2)) + 4u * h + (e & 3u);
            bh[mm][e] = (_Float16)(parity32(k & col) ? -0.25f : 0.25f);
        }
    // Constants the compiler must not fold: the -1 of stage B's remainder (so that value - piece stays a multiply-add
    // and becomes v_fma_mixlo/hi_f16) and the two constants of stage A's second piece (one v_and_or_b32 from registers).
    float minus_one = -1.f;
    asm volatile("" : "+s"(minus_one));
    uint32_t lo_mask = 0x007F007Fu, lo_magic = 0x48004800u;
    asm volatile("" : "+s"(lo_mask));
    asm volatile("" : "+v"(lo_magic));
    // Stage A's products start from minus the bias of the pieces instead of zero: (1152 * 128 + 1024) * 32 / 512 on the
    // lanes tA = 0, nothing elsewhere.  The two vectors live in LDS and are read into the accumulator registers, so
    // the bias costs neither registers nor vector instructions.
    if (t < 32u) bias_tab[t] = t < 16u ? 0.f : -(float)((1152 * 128 + 1024) * 32) * 0x1p-9f;
    const float *const bias_mine = bias_tab + (col == 0u ? 16u : 0u);

    // loads: lane = (column pair, rB bits 0..1), wave = (rB bits 2..4, rA bit 4), register p = rA bits 0..3
    const uint32_t cp = lane & 15u, rl = lane >> 4;
    const uint32_t pitch = (1u << kTileLog2) + a.src_pad; // elements between rows
    const uint32_t rb_mine = rl + 4u * (wave & 7u), ra_mine = 16u * (wave >> 3);
    const uint32_t ld_off = ((32u * ra_mine + rb_mine) * pitch + 2u * cp) * 2u; // bytes
    const uint32_t st_word = cp * kShPairWords + rb_mine * kShRowWords + ra_mine;
    const uint32_t rd_word = wave * kShPairWords + col * kShRowWords + 4u * h;
    uint32_t raw[16];
    // A worker's tile is asked for in four parts (part q = registers 4 q .. 4 q + 3), spread over the arithmetic of the
    // worker before, so that the address unit works through them while the vector unit is busy.
    auto request = [&](uint32_t m, int q) {
        const int16_t *src = static_cast<const int16_t *>(a.src) + (uint64_t)m * a.src_stride + g.origin + (g.origin >> g.ls) * a.src_pad;
        uint32_t off = ld_off;
        asm volatile("" : "+v"(off)); // the zero extension stays next to the loads, which then take the scalar-base form
#pragma unroll
        for (int p = 4 * q; p < 4 * q + 4; ++p) raw[p] = ld_uniform<uint32_t>(src + (uint64_t)(32u * p) * pitch, off);
    };

    float acc[2][16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][r] = acc[1][r] = 0.f;
    const uint32_t sh1 = 30u - 2u * wave; // brings the eps bit of column 2 wave + 1 to bit 31

    // eps word of row tt (32 columns) for worker m, stored where the lanes that need it find their sixteen words 64
    // apart: row = 32 tA + tB goes to 64 (4 (tA / 8) + tA % 4) + 32 ((tA / 4) % 2) + tB
    auto fill_eps_of = [&](uint32_t m) {
        uint32_t tt = t;
        asm volatile("" : "+v"(tt)); // recomputed per worker: nothing of this is held in registers across the loop
        const RngKey key_eps = { a.k0, rk1, kDomainEps, rlo, m };
        const uint64_t i = g.origin + ((uint64_t)tt << kTileLog2);
        uint32_t w[4];
        philox((uint32_t)(i >> 7), key_eps, w);
        const uint32_t sel = (uint32_t)(i >> 5) & 3u;
        const uint32_t ta = tt >> 5;
        epsw[(m & 1u) * 1024u + 64u * (4u * (ta >> 3) + (ta & 3u)) + 32u * ((ta >> 2) & 1u) + (tt & 31u)] =
            sel == 0 ? w[0] : sel == 1 ? w[1] : sel == 2 ? w[2] : w[3];
    };
    float lam_next = a.scales[gb];
    auto process = [&](uint32_t m, auto prefetch) {
        constexpr bool PREFETCH = decltype(prefetch)::value;
        uint32_t *const stage = lds + (m & 1u) * kShStageWords;
        uint32_t *const epsm = epsw + (m & 1u) * 1024u;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            *reinterpret_cast<uint4 *>(stage + st_word + 4 * q) = make_uint4(raw[4 * q], raw[4 * q + 1], raw[4 * q + 2], raw[4 * q + 3]);
        // the next worker's amplitude is asked for ahead of its tile: loads complete in order, so waiting for it
        // later does not wait for the tile
        const float lam_now = lam_next;
        if constexpr (PREFETCH) lam_next = a.scales[(uint64_t)(m + 1) * a.scales_stride + gb];
        // One barrier per worker: the staging buffer written above was last read two workers ago, and every wave has
        // passed the previous worker's barrier only after it was done with those reads.
        __syncthreads();
        uint32_t x[2][8];
#pragma unroll
        for (int mm = 0; mm < 2; ++mm)
#pragma unroll
            for (int e4 = 0; e4 < 2; ++e4) {
                const uint4 q = *reinterpret_cast<const uint4 *>(stage + rd_word + 8 * (2 * mm + e4));
                x[mm][4 * e4] = q.x; x[mm][4 * e4 + 1] = q.y; x[mm][4 * e4 + 2] = q.z; x[mm][4 * e4 + 3] = q.w;
            }
        // the next worker's eps table, while the reads above are on their way; the next barrier publishes it (its
        // buffer was last read one worker ago, before this worker's barrier)
        if constexpr (PREFETCH) fill_eps_of(m + 1);
        const uint32_t cbits = __builtin_amdgcn_readfirstlane(__float_as_uint(lam_now * a.out_coef * 2048.f));
        // The two columns of the wave are interleaved by hand, so that the products of one column run while the
        // vector unit prepares or consumes the other: A0 | pieces 1, A1 | split 0, B0 | split 1, B1 | accumulate 0.
        auto mfma4 = [&](const uint32_t (&p0)[8], const uint32_t (&p1)[8], const mf_v16f &z) -> mf_v16f {
            mf_v16f d = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&p0[0])), bh[0], z, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&p0[4])), bh[1], d, 0, 0, 0);
            d = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&p1[0])), bh[0], d, 0, 0, 0);
            return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(mf_v8h, *reinterpret_cast<const uint4 *>(&p1[4])), bh[1], d, 0, 0, 0);
        };
        // stage A pieces of column 2 wave + j: dword 4 mm + i holds rA = slot(mm, 2 i), slot(mm, 2 i + 1)
        auto pieces = [&](int j, uint32_t (&hi)[8], uint32_t (&lo)[8]) {
#pragma unroll
            for (int mm = 0; mm < 2; ++mm)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t y = __builtin_amdgcn_perm(x[mm][2 * i + 1], x[mm][2 * i], j ? 0x07060302u : 0x05040100u);
                    const sh_s16x2 top = __builtin_bit_cast(sh_s16x2, y) >> 7;
                    hi[4 * mm + i] = __builtin_bit_cast(uint32_t, (sh_u16x2)(__builtin_bit_cast(sh_u16x2, top) + (unsigned short)0x6480));
                    lo[4 * mm + i] = (y & lo_mask) | lo_magic;
                }
        };
        // stage B pieces: register r of d holds rB = 8 (r / 4) + 4 h + r % 4, the k order of bh
        auto split = [&](const mf_v16f &d, uint32_t (&hp)[8], uint32_t (&lp)[8]) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                hp[i] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(d[2 * i], d[2 * i + 1]));
                // remainder = value - first piece, formed and converted in one mixed-precision fma per half
                // (exact: at most ten significant bits)
                typedef _Float16 h2 __attribute__((ext_vector_type(2)));
                const h2 top = __builtin_bit_cast(h2, hp[i]);
                const h2 rest = { (_Float16)fmaf((float)top[0], minus_one, d[2 * i]), (_Float16)fmaf((float)top[1], minus_one, d[2 * i + 1]) };
                lp[i] = __builtin_bit_cast(uint32_t, rest);
            }
        };
        auto bias_vec = [&]() -> mf_v16f {
            asm volatile("" ::: "memory"); // read where it is used, not held in registers
            mf_v16f z;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = *reinterpret_cast<const float4 *>(bias_mine + 4 * q);
                z[4 * q] = v.x; z[4 * q + 1] = v.y; z[4 * q + 2] = v.z; z[4 * q + 3] = v.w;
            }
            return z;
        };
        const mf_v16f zero = { 0 };
        uint32_t pa0[8], pb0[8], pa1[8], pb1[8];
        pieces(0, pa0, pb0);
        const mf_v16f d0 = mfma4(pa0, pb0, bias_vec());
        if constexpr (PREFETCH) request(m + 1, 0);
        __builtin_amdgcn_sched_barrier(0);
        pieces(1, pa1, pb1);
        const mf_v16f d1 = mfma4(pa1, pb1, bias_vec());
        if constexpr (PREFETCH) request(m + 1, 1);
        __builtin_amdgcn_sched_barrier(0);
        split(d0, pa0, pb0);
        const mf_v16f e0 = mfma4(pa0, pb0, zero);
        if constexpr (PREFETCH) request(m + 1, 2);
        __builtin_amdgcn_sched_barrier(0);
        split(d1, pa1, pb1);
        const mf_v16f e1 = mfma4(pa1, pb1, zero);
        if constexpr (PREFETCH) request(m + 1, 3);
        __builtin_amdgcn_sched_barrier(0);
        // register r: row 32 tA + tB with tA = 8 (r / 4) + 4 h + r % 4, tB = lane % 32; columns 2 wave, 2 wave + 1.
        // acc += (+-c) * value: the eps bit goes into the coefficient's sign bit (a flip, whatever the sign was)
        uint32_t ew[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) ew[r] = epsm[64u * r + lane] << sh1;
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[0][r] = fmaf(e0[r], __uint_as_float(__builtin_amdgcn_bitop3_b32(cbits, ew[r] << 1, 0x80000000u, 0x78)), acc[0][r]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r)
            acc[1][r] = fmaf(e1[r], __uint_as_float(__builtin_amdgcn_bitop3_b32(cbits, ew[r], 0x80000000u, 0x78)), acc[1][r]);
    };
#pragma unroll
    for (int q = 0; q < 4; ++q) request(0, q);
    fill_eps_of(0);
    for (uint32_t m = 0; m + 1 < a.M; ++m) process(m, std::true_type{});
    process(a.M - 1, std::false_type{});

    // into the vector-unit kernel's layout LB: reg0 = column bit 0, lanes = (column pair, row bits 0..1),
    // registers = row bits 2..5, waves = row bits 6..9
    __syncthreads(); // the staging buffers are no longer read
    {
        uint2 *const tb = reinterpret_cast<uint2 *>(lds);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const uint32_t row = 32u * (8u * (r >> 2) + 4u * h + (r & 3u)) + col;
            tb[row * kShTransPitch + wave] = make_uint2(__float_as_uint(acc[0][r]), __float_as_uint(acc[1][r]));
        }
    }
    __syncthreads();
    float mean[32];
    {
        const uint2 *const tb = reinterpret_cast<const uint2 *>(lds);
#pragma unroll
        for (int p = 0; p < 16; ++p) {
            const uint32_t row = rl | ((uint32_t)p << 2) | (wave << 6);
            const uint2 d = tb[row * kShTransPitch + cp];
            mean[2 * p] = __uint_as_float(d.x);
            mean[2 * p + 1] = __uint_as_float(d.y);
        }
    }
    __syncthreads(); // the exchange of the tail writes over the transposition buffer
    server_reencode<LV, true>(mean, a, g, tile, rk1, rlo, lds, epsw, red, true);
}

} // namespace fo
