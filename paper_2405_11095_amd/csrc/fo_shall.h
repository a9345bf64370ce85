// Server step when the server shares the workers' eps and all workers share one amplitude per block
// (FO_EPS_SHARED_ALL, a variant the paper does not have).  The server's pre-quantisation vector is
//   H D_eps gbar = H D_eps (lambda / M) D_eps H^T sum_n q_n = (lambda / M) sum_n q_n = (lambda / M)(2 c - M),
// c_i the number of workers whose bit i is set: no transform at all, only a vertical count, the dither of
// Def. 3.2 with amplitude lambda^s, the comparison and the packing (Sec. 4, "Server-to-workers encoding").
// A wave handles 256 consecutive coordinates (four packed words): they share one generator call per lane.
#pragma once
#include "fo_device.h"

namespace fo {

struct ShallArgs {
    const uint64_t *bits_up;   // [M][W]
    uint64_t *dst;             // [planes][W]
    const float *lam;          // [nblocks] the workers' common amplitude
    const float *lam_s;        // [nblocks] the server's amplitude
    uint64_t W;
    uint32_t logb, M, K, planes, dither;
    uint32_t k0, k1, round_lo;
    const unsigned long long *round_dev; // optional: round counter read at run time
    float sqrtb;               // the kernels compare in the unnormalised domain: values and thresholds times sqrt(b)
};

// Vertical count for the 256 coordinates (four packed words 4 q .. 4 q + 3) of a wave: c[s] = number of workers whose
// bit of coordinate 64 s + lane is set.  Lane l first counts the four coordinates of nibble (l & 15) of word (l >> 4):
// the nibble times 0x00204081 has its four bits in the low bit of four bytes, so one add per worker counts four
// coordinates (M <= 64 < 256: no byte overflows); eight lanes read the same 32-bit half word.  Then the byte counts
// move to the lanes of their coordinates: coordinate 64 s + j sits in lane 16 s + j / 4, byte j % 4.
__device__ __forceinline__ void shall_counts(const ShallArgs &a, uint64_t q, uint32_t lane, int32_t (&c)[4])
{
    const uint64_t w = 4 * q + (lane >> 4);
    const uint32_t *const halves = reinterpret_cast<const uint32_t *>(a.bits_up);
    const uint32_t sh = (lane & 7u) * 4u;
    uint32_t cnt = 0u;
    if (w < a.W) {
        const uint32_t *const mine = halves + 2 * w + ((lane >> 3) & 1u);
        for (uint32_t m0 = 0; m0 < a.M; m0 += 8u) { // eight workers' loads in flight at a time
            uint32_t h[8];
#pragma unroll
            for (uint32_t k = 0; k < 8u; ++k) h[k] = (m0 + k < a.M) ? mine[2 * (uint64_t)(m0 + k) * a.W] : 0u;
#pragma unroll
            for (uint32_t k = 0; k < 8u; ++k) cnt += __umul24((h[k] >> sh) & 15u, 0x00204081u) & 0x01010101u;
        }
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint32_t v = (uint32_t)__builtin_amdgcn_ds_bpermute((int)((16u * s + (lane >> 2)) * 4u), (int)cnt);
        c[s] = (int32_t)((v >> ((lane & 3u) * 8u)) & 255u);
    }
}

// ---- measured-norm server amplitude for this mode: ||gbar_block||^2 = (lambda / M)^2 sum_i (2 c_i - M)^2, and the
// sum is an integer, so it is accumulated exactly (and in any order) with 64-bit integer atomics.
static __global__ void k_zero_u64(unsigned long long *p, uint64_t n)
{
    const uint64_t i = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

// Same fetch-and-count as k_shall; sums[j] += sum over block j of (2 c - M)^2.
static __global__ __launch_bounds__(256) void k_shall_sumsq(const ShallArgs a, unsigned long long *sums)
{
    __shared__ unsigned long long part[16];
    const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
    const uint64_t q = (uint64_t)blockIdx.x * 4u + wave;
    int32_t c[4] = { 0, 0, 0, 0 };
    if (4 * q < a.W) shall_counts(a, q, lane, c);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const bool live = 4 * q + s < a.W;
        const int32_t v = live ? 2 * c[s] - (int32_t)a.M : 0;
        uint32_t sq = (uint32_t)(v * v); // at most 64^2 per lane
#pragma unroll
        for (int k = 1; k < 64; k <<= 1) sq += __shfl_xor(sq, k, 64);
        if (lane == 0) part[wave * 4 + s] = sq;
    }
    __syncthreads();
    if (a.logb >= 10u) {
        // the workgroup's 1024 coordinates lie in one block: one atomic for all of them
        if (threadIdx.x == 0) {
            unsigned long long tot = 0;
            for (int i = 0; i < 16; ++i) tot += part[i];
            const uint64_t w0 = (uint64_t)blockIdx.x * 16u;
            if (w0 < a.W) atomicAdd(sums + ((w0 * 64u) >> a.logb), tot);
        }
    } else if (threadIdx.x < 16u) {
        const uint64_t w = (uint64_t)blockIdx.x * 16u + threadIdx.x;
        if (w < a.W) atomicAdd(sums + ((w * 64u) >> a.logb), part[threadIdx.x]);
    }
}

// lambda^s_j = coef * (lambda_j / M) * sqrt(sums[j]),  coef = alpha_s sqrt(ln b / b)
static __global__ void k_shall_scales(const unsigned long long *sums, const float *lam, uint64_t nblocks, uint32_t M, float coef,
                               float *lam_s)
{
    const uint64_t j = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (j < nblocks) lam_s[j] = coef * (lam[j] / (float)M) * (float)sqrt((double)sums[j]);
}

static __global__ __launch_bounds__(256) void k_shall(const ShallArgs a)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint64_t q = (uint64_t)blockIdx.x * 4u + (threadIdx.x >> 6); // group of four words
    if (4 * q >= a.W) return;
    uint32_t rk1, rlo;
    resolve_round(a.k1, a.round_lo, a.round_dev, rk1, rlo);
    int32_t c[4];
    shall_counts(a, q, lane, c);
    float val[4], thr[4];
    uint32_t cnt[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const uint64_t w = 4 * q + s;
        const uint64_t j = w < a.W ? ((w * 64u + lane) >> a.logb) : 0;
        // (2 c - M) / M is exactly +-1 when all workers agree, and lambda sqrt(b) is the very product the threshold
        // below forms when lambda^s = lambda (FO_SERVER_SCALE_SUP): a coordinate at the bound then keeps its sign for
        // every dither
        val[s] = (a.lam[j] * a.sqrtb) * ((float)(2 * c[s] - (int32_t)a.M) / (float)a.M);
        thr[s] = (a.lam_s[j] * a.sqrtb) * 5.9604644775390625e-08f; // 2^-24: u = m 2^-24 with m odd
        cnt[s] = 0u;
    }
    for (uint32_t k = 0; k < a.K; ++k) {
        uint32_t r[4] = { 0u, 0u, 0u, 0u };
        if (a.dither == 0u) {
            const RngKey key = { a.k0, rk1, kDomainDither | (k << 8), rlo, 0xFFFFFFFFu };
            philox((uint32_t)(q << 6) | lane, key, r);
        }
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            float tv = val[s];
            if (a.dither == 0u) tv = fmaf(thr[s], fmaf((float)(r[s] >> 8), 2.f, -16777215.f), tv);
            cnt[s] += (tv >= 0.f) ? 1u : 0u;
        }
    }
    for (uint32_t p = 0; p < a.planes; ++p) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint64_t word = __ballot(((cnt[s] >> p) & 1u) != 0u);
            if (lane == (uint32_t)s && 4 * q + s < a.W) a.dst[(uint64_t)p * a.W + 4 * q + s] = word;
        }
    }
}

} // namespace fo
