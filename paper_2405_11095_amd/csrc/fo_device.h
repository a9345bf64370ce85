// Device-side building blocks of the FO-SGD codec kernels (gfx950, wave64).
//
// Tile model.  Every kernel works on tiles of 2^15 coordinates held entirely in the registers
// of one 512-thread workgroup: 64 values per thread.  A Walsh-Hadamard stage on index bit k is
// a butterfly between two registers of one thread whenever bit k is mapped to the register
// number; the kernels therefore alternate "register rounds" (six stages each, no data
// movement) with exchanges through LDS that remap which index bits live in registers.
// Stages commute, so each kernel visits the bits in the order that suits its memory layout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace fo {

constexpr int kTileLog2 = 15;
constexpr uint32_t kTile = 1u << kTileLog2;
constexpr int kThreads = 512;
constexpr int kV = 64;             // values per thread
constexpr uint32_t kXWords = 16896; // exchange buffer: 128 rows of 128 words padded to 132
constexpr uint32_t kEpsWords = 1024;
constexpr uint32_t kLamWords = 512;
constexpr uint32_t kRedWords = 520;
constexpr uint32_t kLdsWords = kXWords + kEpsWords + kLamWords + kRedWords;

constexpr uint32_t kDomainEps = 1u;
constexpr uint32_t kDomainDither = 2u;

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11): ten rounds of two 32x32->64 multiplies whose high
// halves are mixed with the neighbouring words and the round key; the key advances by two Weyl
// increments per round.  The key schedule is wave-uniform and lives in scalar registers.
// ---------------------------------------------------------------------------------------------
struct RngKey {
    uint32_t k0, k1; // key: seed low word, seed high word xor round high word
    uint32_t c1;     // domain | k << 8
    uint32_t c2;     // round low word
    uint32_t c3;     // party
};

__device__ __forceinline__ void philox(uint32_t counter, const RngKey &key, uint32_t (&out)[4])
{
    uint32_t x0 = counter, x1 = key.c1, x2 = key.c2, x3 = key.c3;
    uint32_t ka = key.k0, kb = key.k1;
#pragma unroll
    for (int i = 0; i < 10; ++i) {
        // full 64-bit products: one v_mad_u64_u32 each instead of a low and a high multiply
        const uint64_t pa = (uint64_t)x0 * 0xD2511F53u;
        const uint64_t pb = (uint64_t)x2 * 0xCD9E8D57u;
        // three-input xor (truth table 0x96) in one v_bitop3_b32
        x0 = __builtin_amdgcn_bitop3_b32((uint32_t)(pb >> 32), x1, ka, 0x96);
        x2 = __builtin_amdgcn_bitop3_b32((uint32_t)(pa >> 32), x3, kb, 0x96);
        x1 = (uint32_t)pb;
        x3 = (uint32_t)pa;
        ka += 0x9E3779B9u;
        kb += 0xBB67AE85u;
    }
    out[0] = x0; out[1] = x1; out[2] = x2; out[3] = x3;
}

// The round counter enters the generator key (low word as counter word 2, high word xored into key word 1).
// It is either fixed at launch (dev == nullptr: k1_in already holds the xor) or read from device memory when
// the kernel runs, so that a captured graph can be replayed for one round after the other.
__device__ __forceinline__ void resolve_round(uint32_t k1_in, uint32_t lo_in, const unsigned long long *dev, uint32_t &k1,
                                              uint32_t &lo)
{
    k1 = k1_in;
    lo = lo_in;
    if (dev) {
        const unsigned long long r = *dev;
        lo = (uint32_t)r;
        k1 = k1_in ^ (uint32_t)(r >> 32);
    }
}

// ---------------------------------------------------------------------------------------------
// Small helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void wave_sync()
{
    // Orders LDS traffic between lanes of one wave: the LDS queue of a wave is in order, the
    // fences keep the compiler from moving accesses across this point.
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float flip_if(float x, uint32_t bit) // bit in {0,1}
{
    return __uint_as_float(__float_as_uint(x) ^ (bit << 31));
}
// x with its sign flipped when bit 31 of w is set: x ^ (w & 0x80000000) as one three-input operation
__device__ __forceinline__ float flip_by_bit31(float x, uint32_t w)
{
    return __uint_as_float(__builtin_amdgcn_bitop3_b32(__float_as_uint(x), w, 0x80000000u, 0x78));
}

template <typename T, int BIT, int V = kV>
__device__ __forceinline__ void bfly(T (&v)[V])
{
    static_assert((1 << BIT) < V, "stage bit outside the register index");
#pragma unroll
    for (int r = 0; r < V; ++r)
        if (!(r & (1 << BIT))) {
            const T a = v[r], b = v[r | (1 << BIT)];
            v[r] = a + b;
            v[r | (1 << BIT)] = a - b;
        }
}

__device__ __forceinline__ float wave_sum(float s, int steps) // butterfly sum over 2^steps lanes
{
#pragma unroll
    for (int k = 0; k < 6; ++k)
        if (k < steps) s += __shfl_xor(s, 1 << k, 64);
    return s;
}

// Compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// v_writelane_b32 as the compiler's own intrinsic (this toolchain has no clang builtin for it, so the LLVM
// intrinsic is bound by name).  Unlike inline assembly, the compiler sees the instruction and inserts the wait
// states gfx950 needs between a vector compare that writes a scalar register pair and a vector instruction that
// reads it (two; back to back the lane write can pick up the register's previous contents).
extern "C" __device__ int fo_llvm_writelane(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");

// Returns v with lane LANE replaced by the wave-uniform value s (every other lane keeps its own).
template <int LANE>
__device__ __forceinline__ uint32_t write_lane(uint32_t v, uint32_t s)
{
    return (uint32_t)fo_llvm_writelane((int)s, LANE, (int)v);
}

// One Walsh-Hadamard stage on lane bit 5 (partner = lane ^ 32).  v_permlane32_swap trades the
// upper half-wave of its first operand with the lower half-wave of its second, which brings both
// ends of a butterfly into one lane; a second swap restores the layout.
template <typename T, int V>
__device__ __forceinline__ void bfly_lane5(T (&v)[V])
{
#pragma unroll
    for (int k = 0; k < V / 2; ++k) {
        uint32_t a = __builtin_bit_cast(uint32_t, v[k]), b = __builtin_bit_cast(uint32_t, v[k + V / 2]);
        auto r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
        const T x = __builtin_bit_cast(T, (uint32_t)r[0]), y = __builtin_bit_cast(T, (uint32_t)r[1]);
        a = __builtin_bit_cast(uint32_t, (T)(x + y));
        b = __builtin_bit_cast(uint32_t, (T)(x - y));
        r = __builtin_amdgcn_permlane32_swap(a, b, false, false);
        v[k] = __builtin_bit_cast(T, (uint32_t)r[0]);
        v[k + V / 2] = __builtin_bit_cast(T, (uint32_t)r[1]);
    }
}

// Swap register bit 5 with lane bit 5: afterwards v[k] of the upper half-wave and v[k+32] of
// the lower half-wave have traded places.
template <typename T>
__device__ __forceinline__ void swap_reg5_lane5(T (&v)[kV])
{
#pragma unroll
    for (int k = 0; k < 32; ++k) {
        const uint32_t lo = __builtin_bit_cast(uint32_t, v[k]);
        const uint32_t hi = __builtin_bit_cast(uint32_t, v[k + 32]);
        // v_permlane32_swap: lanes 32..63 of the first operand trade with lanes 0..31 of the second
        const auto r = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
        v[k] = __builtin_bit_cast(T, (uint32_t)r[0]);
        v[k + 32] = __builtin_bit_cast(T, (uint32_t)r[1]);
    }
}

} // namespace fo
