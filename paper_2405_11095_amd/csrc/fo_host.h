// Host-side internals shared by the library's translation units (fo_api.hip, fo_enc.hip, fo_enc_stats.hip,
// fo_dec.hip, fo_srv.hip): the plan, the kernel launcher with its optional event bracketing, argument-block
// builders and the launch sequences' declarations.  The library is split into several translation units only
// so that they compile side by side; every step of the codec runs in the kernels of fo_contig.h, fo_strided.h,
// fo_declow.h, fo_server_tile.h, fo_server_high.h and fo_shall.h.
#pragma once
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <type_traits>

#include "../../include/fo.h"
#include "fo_strided.h"
#include "fo_declow.h"
#include "fo_server_tile.h"
#include "fo_shall.h"

// Kernel identities for the optional per-kernel timing (fo_profile_begin / fo_profile_end).
enum KernelId {
    KID_ENC_SINGLE = 0, // k_contig<IN_GRAD,OUT_PACK>
    KID_ENC_HIGH,       // k_strided<ENC_FIRST>
    KID_ENC_MID,        // k_strided<MID_F32>
    KID_ENC_LOW,        // k_contig<IN_F32,OUT_PACK>
    KID_DEC_SINGLE,     // k_contig<IN_BITS,OUT_F32>
    KID_DEC_LOW,        // k_declow (k_contig<IN_BITS,OUT_I32> for three-pass transforms)
    KID_DEC_MID,        // k_strided<MID_I32>
    KID_DEC_HIGH,       // k_strided<DEC_LAST>
    KID_SERVER_HIGH,    // k_strided<SERVER> / k_strided<SHARED>
    KID_SERVER_MFMA,    // k_server_mfma
    KID_COUNT_LOW,      // k_contig<IN_COUNT,*>
    KID_SERVER_TILE,    // k_mean_mfma
    KID_SHALL,          // k_shall
    KID_ENC_PAIR,       // k_contig_pair
    KID_DEC_PAIR,       // k_decode_pair
    KID_SCALES,         // k_finalize_scales / k_fill_scales / k_server_scales
    KID_COUNT
};
inline const char *const kKernelNames[KID_COUNT] = {
    "k_contig<IN_GRAD,OUT_PACK>", "k_strided<ENC_FIRST>", "k_strided<MID_F32>", "k_contig<IN_F32,OUT_PACK>",
    "k_decode_tile",  "k_declow", "k_strided<MID_I32>", "k_strided<DEC_LAST>",
    "k_strided<SERVER>", "k_server_mfma", "k_contig<IN_COUNT>", "k_mean_mfma", "k_shall", "k_contig_pair", "k_decode_pair", "scale kernels",
};

struct Profiler {
    bool on = false;
    static constexpr int kMax = 8192;
    hipEvent_t *ev = nullptr; // 2 * kMax events
    int *kid = nullptr;       // kMax entries, allocated with the events
    int used = 0;
    int only = -1; // >= 0: bracket launches of this kernel only
};


// ---------------------------------------------------------------------------------------------
// Plan
// ---------------------------------------------------------------------------------------------
struct fo_plan {
    fo_params p;
    uint32_t logb;       // log2 of the transform length
    uint64_t b, nblocks, ntot, W, ntiles;
    uint32_t S;          // stages done by the contiguous kernel
    uint32_t npass;      // strided passes: 0, 1 or 2
    uint32_t hb[2];      // stages of each strided pass (pass 0 is adjacent to the contiguous tile)
    uint32_t planes;     // bit planes of the downlink message: ceil(log2(K + 1))
    uint32_t num_cus;    // compute units of the device the plan was made on
    uint32_t pad32, pad16; // elements between the 2^15-element rows of the fp32 / int16 intermediates (two-pass transforms)
    bool server_mfma;    // blocks of 2^25: the server pass on the matrix cores (off: the vector-unit kernel, same results)
    float coef_lambda, sqrtb, rsqrtb, coef_s;
    float coef_lambda_s; // alpha_s sqrt(ln b / b): measured-norm rule for the server
    // scratch (device)
    char *scratch;
    size_t scratch_bytes;
    float *buf_a;        // [M][ntot] 4-byte intermediates (transform lengths above 2^15)
    float *buf_b;        // [ntot] mean gradient / server intermediate
    float *buf_c;        // [ntot] second intermediate for three-pass transforms, else NULL
    float *partials;     // [M][ntiles]
    uint64_t *bits_up;   // [M][W]
    float *scales_up;    // [M][nblocks]
    uint64_t *bits_down; // [planes][W]
    float *scales_down;  // [nblocks]
    unsigned long long *blk_sums; // [nblocks] integer sums of squares (all-shared eps with the measured-norm rule)
    fo_stats *stats;     // device, optional
    const unsigned long long *round_dev; // device, set for the duration of fo_step_dev_round
    Profiler prof;
};

namespace fo_host {

using namespace fo;

extern thread_local char g_hip_err[256]; // text of the last HIP error on this thread (fo_last_hip_error)

inline bool hip_ok(hipError_t e, const char *what)
{
    if (e == hipSuccess) return true;
    std::snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
    return false;
}

inline bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

struct Rng {
    uint32_t k0, k1, round_lo;
    const unsigned long long *round_dev;
};
inline Rng rng_of(const fo_plan *pl, uint64_t round)
{
    // with a device-side round counter the kernels finish the key themselves (resolve_round)
    if (pl->round_dev) return { (uint32_t)pl->p.seed, (uint32_t)(pl->p.seed >> 32), 0u, pl->round_dev };
    return { (uint32_t)pl->p.seed, (uint32_t)(pl->p.seed >> 32) ^ (uint32_t)(round >> 32), (uint32_t)round, nullptr };
}

// Host-side guard against launching a kernel with a pointer it will dereference left unset.
inline bool args_ok(const ContigArgs &c, const PtrTab &tab, int kid)
{
    const bool grad_in = kid == KID_ENC_SINGLE || kid == KID_ENC_PAIR;
    if (!c.dst) return false;
    if (kid == KID_ENC_PAIR && (c.logb != 16 || c.S != 15)) return false;
    if (grad_in ? (c.use_tab ? !tab.p[0] : !c.src) : !c.src) return false;
    const bool needs_scales = kid == KID_ENC_SINGLE || kid == KID_ENC_PAIR || kid == KID_ENC_LOW || kid == KID_DEC_SINGLE;
    if (kid == KID_COUNT_LOW && (c.M < 1 || c.M > FO_MAX_WORKERS)) return false;
    return !needs_scales || c.scales != nullptr;
}
inline bool args_ok(const ContigArgs &c, int kid) // k_declow, k_decode_tile
{
    if (kid == KID_DEC_PAIR) return c.src && c.dst && c.scales && c.logb == 16;
    return c.src && c.dst && (kid != KID_DEC_SINGLE || (c.scales && c.S >= 6 && c.S <= 15));
}
inline bool args_ok(const ShallArgs &z, int)
{
    return z.bits_up && z.dst && z.lam && z.lam_s && z.M >= 1 && z.M <= FO_MAX_WORKERS && z.K >= 1 && z.planes >= 1;
}
inline bool args_ok(const ShallArgs &z, unsigned long long *sums, int kid) { return sums && args_ok(z, kid); }
inline bool args_ok(const ServerTileArgs &s, uint32_t ntiles, int kid);
inline bool args_ok(const ServerTileArgs &s, int)
{
    return s.enc.src && s.bits_up && s.scales_up && s.M >= 1 && s.M <= FO_MAX_WORKERS && s.enc.S >= 6 && s.enc.S <= 15;
}
inline bool args_ok(const ServerTileArgs &s, uint32_t ntiles, int kid) { return ntiles >= 1 && args_ok(s, kid); }
inline bool args_ok(const StridedArgs &s, const PtrTab &tab, int kid)
{
    if (!s.dst) return false;
    if (kid == KID_ENC_HIGH ? (s.use_tab ? !tab.p[0] : !s.src) : !s.src) return false;
    if (kid == KID_ENC_HIGH && !s.partials) return false;
    if ((kid == KID_DEC_HIGH || kid == KID_SERVER_HIGH || kid == KID_SERVER_MFMA) && !s.scales) return false;
    return s.hb >= 1 && s.hb <= 10 && s.ls >= (uint32_t)kTileLog2;
}
template <typename... Args>
inline bool args_ok(const Args &...) { return true; }

// Enqueue one kernel; with profiling on, bracket it with two HIP events on the same stream.
template <typename Kern, typename... Args>
int launch(fo_plan *pl, int kid, Kern kernel, dim3 grid, dim3 block, hipStream_t st, Args... args)
{
    if (!args_ok(args..., kid)) {
        std::snprintf(g_hip_err, sizeof(g_hip_err), "internal: unset kernel argument for %s", kKernelNames[kid]);
        return FO_EHIP;
    }
    Profiler &pf = pl->prof;
    const bool rec = pf.on && (pf.only < 0 || pf.only == kid) && pf.used < Profiler::kMax;
    if (rec && !hip_ok(hipEventRecord(pf.ev[2 * pf.used], st), "hipEventRecord")) return FO_EHIP;
    hipLaunchKernelGGL(kernel, grid, block, 0, st, args...);
    if (!hip_ok(hipGetLastError(), kKernelNames[kid])) return FO_EHIP;
    if (rec) {
        if (!hip_ok(hipEventRecord(pf.ev[2 * pf.used + 1], st), "hipEventRecord")) return FO_EHIP;
        pf.kid[pf.used++] = kid;
    }
    return FO_OK;
}
#define FO_TRY(expr)               \
    do {                           \
        const int rc_ = (expr);    \
        if (rc_) return rc_;       \
    } while (0)

// Strided kernels come in a generic form and one compiled for ten stages next to the contiguous tile.
template <int MODE, bool IN16 = false>
int launch_strided(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const StridedArgs &s, const PtrTab &tab)
{
    constexpr int LV = (MODE == SM_SERVER || MODE == SM_SHARED || MODE == SM_ENC_FIRST) ? 5 : 6;
    if (s.hb == 10 && s.ls == (uint32_t)kTileLog2)
        return launch(pl, kid, k_strided<MODE, 10, IN16, LV>, grid, dim3(SL<LV>::T), st, s, tab);
    return launch(pl, kid, k_strided<MODE, 0, IN16, LV>, grid, dim3(SL<LV>::T), st, s, tab);
}

inline StridedArgs strided_base(const fo_plan *pl, const Rng &r, uint32_t pass)
{
    StridedArgs s;
    std::memset(&s, 0, sizeof(s));
    s.hb = pl->hb[pass];
    s.ls = pass == 0 ? (uint32_t)kTileLog2 : (uint32_t)kTileLog2 + pl->hb[0];
    s.logb = pl->logb;
    s.k0 = r.k0; s.k1 = r.k1; s.round_lo = r.round_lo; s.round_dev = r.round_dev;
    s.len_in = s.len_out = pl->ntot;
    return s;
}

inline ContigArgs contig_base(const fo_plan *pl, const Rng &r)
{
    ContigArgs c;
    std::memset(&c, 0, sizeof(c));
    c.W = pl->W;
    c.nblocks = pl->nblocks;
    c.S = pl->S;
    c.logb = pl->logb;
    c.dither = pl->p.dither;
    c.k0 = r.k0; c.k1 = r.k1; c.round_lo = r.round_lo; c.round_dev = r.round_dev;
    c.coef_lambda = pl->coef_lambda;
    c.sqrtb = pl->sqrtb;
    c.len_in = c.len_out = pl->ntot;
    c.K = 1; c.planes = 1;
    return c;
}
// Messages of the server carry the K-fold quantiser's counts (Def. 3.2); workers' messages are plain signs.
// Also points the encode at the party's diagnostic counters when a stats block is attached.
inline void set_quantiser(ContigArgs &c, const fo_plan *pl, uint32_t party)
{
    c.K = party == FO_PARTY_SERVER ? pl->p.K : 1u;
    c.planes = party == FO_PARTY_SERVER ? pl->planes : 1u;
    if (pl->stats) {
        const uint32_t at = party == FO_PARTY_SERVER ? FO_MAX_WORKERS : party;
        c.stat_clipped = pl->stats->clipped + at;
        c.stat_near = pl->stats->near_tie + at;
    }
}

constexpr uint32_t kPartyAllWorkers = 0xFFFFFFFEu;
// Which eps stream a party uses: its own, or the common one of the workers in shared-eps mode.
inline uint32_t eps_party_of(const fo_plan *pl, uint32_t party)
{
    if (pl->p.eps_mode == FO_EPS_INDEPENDENT) return party;
    if (party == FO_PARTY_SERVER && pl->p.eps_mode == FO_EPS_SHARED_WORKERS) return party;
    return kPartyAllWorkers;
}


// ---------------------------------------------------------------------------------------------
// Launch sequences (one translation unit each)
// ---------------------------------------------------------------------------------------------

// Row padding of the intermediates of two-pass transforms: one 128-byte line (see StridedArgs).
constexpr uint32_t kRowPad32 = 32, kRowPad16 = 64;

// fo_api.hip: the small amplitude kernels
int launch_finalize_scales(fo_plan *pl, hipStream_t st, uint32_t nslots, float coef, float *scales, uint64_t scales_stride);
int launch_fill_scales(fo_plan *pl, hipStream_t st, uint32_t nslots, float *scales, uint64_t scales_stride, float value);
int launch_server_scales(fo_plan *pl, hipStream_t st, const float *scales_up, float *scales_down);
int launch_common_scales(fo_plan *pl, hipStream_t st, float *scales, uint32_t nslots);

// fo_enc.hip / fo_enc_stats.hip: the dither + sign + pack kernels, without / with the diagnostic counters
template <int IN, bool STATS>
int launch_pack_s(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab);
extern template int launch_pack_s<IN_GRAD, false>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
extern template int launch_pack_s<IN_F32, false>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
extern template int launch_pack_s<IN_GRAD, true>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
extern template int launch_pack_s<IN_F32, true>(fo_plan *, int, dim3, hipStream_t, const ContigArgs &, const PtrTab &);
// The variants with the diagnostic counters compiled in run only while a stats block is attached.
template <int IN>
inline int launch_pack(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    if (c.stat_clipped) return launch_pack_s<IN, true>(pl, kid, grid, st, c, tab);
    return launch_pack_s<IN, false>(pl, kid, grid, st, c, tab);
}
int launch_encode(fo_plan *pl, const PtrTab *tab, const float *src, uint64_t src_stride, uint64_t len_in,
                  uint32_t nslots, uint32_t party0, uint64_t round, bool scales_given, uint64_t *bits,
                  uint64_t bits_stride, float *scales, uint64_t scales_stride, float *tmp, uint64_t tmp_stride,
                  hipStream_t st, bool common = false);

// fo_dec.hip
int launch_declow(fo_plan *pl, dim3 grid, hipStream_t st, const ContigArgs &c);
int launch_decode(fo_plan *pl, const uint64_t *bits, const float *scales, uint64_t round, uint32_t party,
                  float *out, uint64_t len_out, uint32_t store_mode, float out_coef, float delta, float *tmp,
                  hipStream_t st);

// fo_srv.hip
int launch_server(fo_plan *pl, const uint64_t *bits_up, const float *scales_up, uint64_t round, uint64_t *bits_down,
                  float *scales_down, float *gbar_or_null, hipStream_t st);

} // namespace fo_host
