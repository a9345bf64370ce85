// C ABI of the FO-SGD codec (declared in include/fo.h): argument checks, plan scratch and kernel
// launch sequences.  Every step of the codec runs in the kernels of fo_contig.h, fo_strided.h, fo_declow.h,
// fo_server_tile.h and fo_shall.h.
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

using namespace fo;

namespace {

thread_local char g_hip_err[256] = "";

bool hip_ok(hipError_t e, const char *what)
{
    if (e == hipSuccess) return true;
    std::snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
    return false;
}

// ---------------------------------------------------------------------------------------------
// Small kernels
// ---------------------------------------------------------------------------------------------

// lambda_j = coef * sqrt(sum of the tile partials of block j)   (amplitude of Thm 5.5, B = ||g_block||)
__global__ __launch_bounds__(256) void k_finalize_scales(const float *partials, uint64_t ntiles, uint32_t tiles_per_block,
                                                          float coef, float *scales, uint64_t scales_stride)
{
    __shared__ double red[256];
    const uint32_t j = blockIdx.x, slot = blockIdx.y, t = threadIdx.x;
    const float *p = partials + (uint64_t)slot * ntiles + (uint64_t)j * tiles_per_block;
    double s = 0.0;
    for (uint32_t k = t; k < tiles_per_block; k += 256) s += (double)p[k];
    red[t] = s;
    __syncthreads();
    for (uint32_t h = 128; h > 0; h >>= 1) {
        if (t < h) red[t] += red[t + h];
        __syncthreads();
    }
    if (t == 0) scales[slot * scales_stride + j] = coef * (float)sqrt(red[0]);
}

__global__ void k_fill_scales(float *scales, uint64_t scales_stride, uint64_t nblocks, float value)
{
    const uint64_t j = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (j < nblocks) scales[blockIdx.y * scales_stride + j] = value;
}

// lambda^s_j = coef_s * max_n lambda_{n,j}   (Thm 5.5: lambda^s = alpha_s * lambda * sqrt(log n))
__global__ void k_server_scales(const float *scales_up, uint64_t nblocks, uint32_t M, float coef_s, float *scales_down)
{
    const uint64_t j = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (j >= nblocks) return;
    float m = 0.f;
    bool nan = false;
    for (uint32_t n = 0; n < M; ++n) {
        const float l = scales_up[(uint64_t)n * nblocks + j];
        nan |= (l != l);
        m = fmaxf(m, l);
    }
    scales_down[j] = nan ? __builtin_nanf("") : coef_s * m;
}

// Shared-eps mode: every worker quantises with the largest of the workers' amplitudes, per block.
__global__ void k_common_scales(float *scales, uint64_t nblocks, uint32_t M)
{
    const uint64_t j = blockIdx.x * (uint64_t)blockDim.x + threadIdx.x;
    if (j >= nblocks) return;
    float m = 0.f;
    bool nan = false;
    for (uint32_t n = 0; n < M; ++n) {
        const float l = scales[(uint64_t)n * nblocks + j];
        nan |= (l != l);
        m = fmaxf(m, l);
    }
    if (nan) m = __builtin_nanf("");
    for (uint32_t n = 0; n < M; ++n) scales[(uint64_t)n * nblocks + j] = m;
}

bool aligned(const void *p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

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
    KID_COUNT_LOW,      // k_contig<IN_COUNT,*>
    KID_SERVER_TILE,    // k_mean_tile
    KID_SHALL,          // k_shall
    KID_ENC_PAIR,       // k_contig_pair
    KID_DEC_PAIR,       // k_decode_pair
    KID_SCALES,         // k_finalize_scales / k_fill_scales / k_server_scales
    KID_COUNT
};
const char *const kKernelNames[KID_COUNT] = {
    "k_contig<IN_GRAD,OUT_PACK>", "k_strided<ENC_FIRST>", "k_strided<MID_F32>", "k_contig<IN_F32,OUT_PACK>",
    "k_decode_tile",  "k_declow", "k_strided<MID_I32>", "k_strided<DEC_LAST>",
    "k_strided<SERVER>", "k_contig<IN_COUNT>", "k_mean_tile", "k_shall", "k_contig_pair", "k_decode_pair", "scale kernels",
};

struct Profiler {
    bool on = false;
    static constexpr int kMax = 8192;
    hipEvent_t *ev = nullptr; // 2 * kMax events
    int *kid = nullptr;       // kMax entries, allocated with the events
    int used = 0;
    int only = -1; // >= 0: bracket launches of this kernel only
};

} // namespace

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

extern "C" const char *fo_last_hip_error(void) { return g_hip_err; }

namespace {

// Validates the parameters and fills in everything of a plan that is host arithmetic (no device memory).
int plan_geometry(const fo_params &q, fo_plan *pl)
{
    if (q.d < 1 || q.M < 1 || q.M > FO_MAX_WORKERS) return FO_EINVAL;
    if (q.block_log2 != 0 && (q.block_log2 < 6 || q.block_log2 > 30)) return FO_EINVAL;
    if (q.K < 1 || q.K > FO_MAX_K) return FO_EINVAL;
    if (q.dither != FO_DITHER_UNIFORM && q.dither != FO_DITHER_NONE) return FO_EINVAL;
    if (q.scale_rule != FO_SCALE_BOUND && q.scale_rule != FO_SCALE_L2) return FO_EINVAL;
    if (q.eps_mode != FO_EPS_INDEPENDENT && q.eps_mode != FO_EPS_SHARED_WORKERS && q.eps_mode != FO_EPS_SHARED_ALL)
        return FO_EINVAL;
    if (!(q.alpha >= 2.f) || !(q.alpha_s >= 2.f)) return FO_EINVAL;
    if (q.scale_rule == FO_SCALE_BOUND && !(q.B > 0.f)) return FO_EINVAL;
    if (q.server_scale != FO_SERVER_SCALE_THM && q.server_scale != FO_SERVER_SCALE_L2) return FO_EINVAL;

    pl->p = q;
    pl->stats = nullptr;
    pl->round_dev = nullptr;
    if (q.block_log2 == 0) {
        uint32_t k = 6;
        while (((uint64_t)1 << k) < q.d) ++k;
        if (k > 30) return FO_EINVAL;
        pl->logb = k;
        pl->nblocks = 1;
    } else {
        pl->logb = q.block_log2;
        pl->nblocks = (q.d + (((uint64_t)1 << pl->logb) - 1)) >> pl->logb;
    }
    pl->b = (uint64_t)1 << pl->logb;
    pl->ntot = pl->b * pl->nblocks;
    if (pl->ntot > ((uint64_t)1 << 32)) return FO_EINVAL;
    pl->W = pl->ntot / 64;
    pl->ntiles = (pl->ntot + kTile - 1) / kTile;
    pl->S = pl->logb < (uint32_t)kTileLog2 ? pl->logb : (uint32_t)kTileLog2;
    const uint32_t high = pl->logb - pl->S;
    pl->npass = high == 0 ? 0 : (high <= 10 ? 1 : 2);
    pl->hb[0] = pl->npass == 2 ? (high + 1) / 2 : high;
    pl->hb[1] = high - pl->hb[0];
    if (q.eps_mode != FO_EPS_INDEPENDENT && pl->npass == 2) return FO_EINVAL; // shared eps: not built for b > 2^25
    pl->planes = 0;
    while ((q.K >> pl->planes) != 0) ++pl->planes;
    // the decode side carries K b / 2 at most in int32 between its passes
    if (q.K > 1 && pl->npass > 0 && (uint64_t)q.K * (pl->b / 2) >= ((uint64_t)1 << 31)) return FO_EINVAL;
    const double bd = (double)pl->b;
    pl->coef_lambda = (float)((double)q.alpha * std::sqrt(std::log(bd) / bd));
    pl->sqrtb = (float)std::sqrt(bd);
    pl->rsqrtb = (float)(1.0 / std::sqrt(bd));
    pl->coef_s = (float)((double)q.alpha_s * std::sqrt(std::log(bd)));
    pl->coef_lambda_s = (float)((double)q.alpha_s * std::sqrt(std::log(bd) / bd));
    return FO_OK;
}

} // namespace

extern "C" int fo_plan_create(const fo_params *params, fo_plan **out)
{
    if (!params || !out) return FO_EINVAL;
    *out = nullptr;
    const fo_params &q = *params;
    fo_plan *pl = new (std::nothrow) fo_plan();
    if (!pl) return FO_ENOMEM;
    {
        const int rc = plan_geometry(q, pl);
        if (rc) { delete pl; return rc; }
    }

    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    const size_t sz_a = pl->npass ? up((size_t)q.M * pl->ntot * 4) : 0;
    const size_t sz_b = up(pl->ntot * 4);
    const size_t sz_c = pl->npass == 2 ? up(pl->ntot * 4) : 0;
    const size_t sz_part = up((size_t)q.M * pl->ntiles * 4);
    const size_t sz_bu = up((size_t)q.M * pl->W * 8), sz_su = up((size_t)q.M * pl->nblocks * 4);
    const size_t sz_bd = up((size_t)pl->planes * pl->W * 8), sz_sd = up(pl->nblocks * 4);
    const size_t sz_bs = up(pl->nblocks * 8);
    pl->scratch_bytes = sz_a + sz_b + sz_c + sz_part + sz_bu + sz_su + sz_bd + sz_sd + sz_bs;
    void *mem = nullptr;
    hipError_t e = hipMalloc(&mem, pl->scratch_bytes);
    if (e != hipSuccess) {
        hip_ok(e, "hipMalloc(plan scratch)");
        delete pl;
        return e == hipErrorOutOfMemory ? FO_ENOMEM : FO_EHIP;
    }
    char *c = static_cast<char *>(mem);
    pl->scratch = c;
    pl->buf_a = sz_a ? reinterpret_cast<float *>(c) : nullptr; c += sz_a;
    pl->buf_b = reinterpret_cast<float *>(c); c += sz_b;
    pl->buf_c = sz_c ? reinterpret_cast<float *>(c) : nullptr; c += sz_c;
    pl->partials = reinterpret_cast<float *>(c); c += sz_part;
    pl->bits_up = reinterpret_cast<uint64_t *>(c); c += sz_bu;
    pl->scales_up = reinterpret_cast<float *>(c); c += sz_su;
    pl->bits_down = reinterpret_cast<uint64_t *>(c); c += sz_bd;
    pl->scales_down = reinterpret_cast<float *>(c); c += sz_sd;
    pl->blk_sums = reinterpret_cast<unsigned long long *>(c);
    *out = pl;
    return FO_OK;
}

extern "C" void fo_plan_destroy(fo_plan *plan)
{
    if (!plan) return;
    if (plan->scratch) (void)hipFree(plan->scratch);
    if (plan->prof.ev) {
        for (int i = 0; i < 2 * Profiler::kMax; ++i) (void)hipEventDestroy(plan->prof.ev[i]);
        delete[] plan->prof.ev;
        delete[] plan->prof.kid;
    }
    delete plan;
}

extern "C" size_t fo_padded_len(const fo_plan *p) { return p ? p->ntot : 0; }
extern "C" size_t fo_packed_words(const fo_plan *p) { return p ? p->W : 0; }
extern "C" size_t fo_num_scales(const fo_plan *p) { return p ? p->nblocks : 0; }
extern "C" size_t fo_block_len(const fo_plan *p) { return p ? p->b : 0; }
extern "C" size_t fo_downlink_planes(const fo_plan *p) { return p ? p->planes : 0; }
extern "C" size_t fo_scratch_bytes(const fo_plan *p) { return p ? p->scratch_bytes : 0; }

// ---------------------------------------------------------------------------------------------
// Launch sequences
// ---------------------------------------------------------------------------------------------
namespace {

struct Rng {
    uint32_t k0, k1, round_lo;
    const unsigned long long *round_dev;
};
Rng rng_of(const fo_plan *pl, uint64_t round)
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
inline bool args_ok(const ServerTileArgs &s, int)
{
    return s.enc.src && s.bits_up && s.scales_up && s.M >= 1 && s.M <= FO_MAX_WORKERS && s.enc.S >= 6 && s.enc.S <= 15;
}
inline bool args_ok(const StridedArgs &s, const PtrTab &tab, int kid)
{
    if (!s.dst) return false;
    if (kid == KID_ENC_HIGH ? (s.use_tab ? !tab.p[0] : !s.src) : !s.src) return false;
    if (kid == KID_ENC_HIGH && !s.partials) return false;
    if ((kid == KID_DEC_HIGH || kid == KID_SERVER_HIGH) && !s.scales) return false;
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

// The packing kernels are compiled per (dither on/off, transform length below 256).
template <int IN, bool STATS>
int launch_pack_s(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    const bool dither = c.dither == FO_DITHER_UNIFORM, small = c.S < 8;
    const dim3 block(kThreads);
    if (c.K > 1) { // the K-fold quantiser of the server's message
        if (dither && small) return launch(pl, kid, k_contig<IN, OUT_PACK, true, true, 0, true, STATS>, grid, block, st, c, tab);
        if (dither) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 0, true, STATS>, grid, block, st, c, tab);
        return launch(pl, kid, k_contig<IN, OUT_PACK, false, false, 0, true, STATS>, grid, block, st, c, tab);
    }
    if (dither && c.S == 15) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 15, false, STATS>, grid, block, st, c, tab);
    if constexpr (IN == IN_GRAD && !STATS) {
        // block lengths of the blocked workload, compiled for their stage count; tiles that lie inside the input
        // whole go to a variant without the per-chunk end-of-input checks
        if (dither && (c.S == 10 || c.S == 12 || c.S == 14)) {
            const uint64_t full64 = c.len_in >> kTileLog2;
            const uint32_t nfull = (uint32_t)(full64 < grid.x ? full64 : grid.x);
            ContigArgs cc = c;
            auto go = [&](auto sc, auto guarded, uint32_t tile0, uint32_t ntile) -> int {
                cc.tile0 = tile0;
                return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, decltype(sc)::value, false, false, decltype(guarded)::value>,
                              dim3(ntile, grid.y), block, st, cc, tab);
            };
            auto both = [&](auto sc) -> int {
                if (nfull) FO_TRY(go(sc, std::false_type{}, 0u, nfull));
                if (nfull < grid.x) FO_TRY(go(sc, std::true_type{}, nfull, grid.x - nfull));
                return FO_OK;
            };
            if (c.S == 10) return both(std::integral_constant<int, 10>{});
            if (c.S == 12) return both(std::integral_constant<int, 12>{});
            return both(std::integral_constant<int, 14>{});
        }
    }
    if (dither && small) return launch(pl, kid, k_contig<IN, OUT_PACK, true, true, 0, false, STATS>, grid, block, st, c, tab);
    if (dither) return launch(pl, kid, k_contig<IN, OUT_PACK, true, false, 0, false, STATS>, grid, block, st, c, tab);
    return launch(pl, kid, k_contig<IN, OUT_PACK, false, false, 0, false, STATS>, grid, block, st, c, tab);
}
// The variants with the diagnostic counters compiled in run only while a stats block is attached.
template <int IN>
int launch_pack(fo_plan *pl, int kid, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    if (c.stat_clipped) return launch_pack_s<IN, true>(pl, kid, grid, st, c, tab);
    return launch_pack_s<IN, false>(pl, kid, grid, st, c, tab);
}

// Encode of blocks of 2^16 coordinates in one pass.
int launch_pair(fo_plan *pl, dim3 grid, hipStream_t st, const ContigArgs &c, const PtrTab &tab)
{
    const bool dither = c.dither == FO_DITHER_UNIFORM;
    const dim3 block(2 * kThreads);
    if (c.K > 1) {
        if (dither) return launch(pl, KID_ENC_PAIR, k_contig_pair<true, true>, grid, block, st, c, tab);
        return launch(pl, KID_ENC_PAIR, k_contig_pair<false, true>, grid, block, st, c, tab);
    }
    if (dither) {
        // blocks that lie inside the input whole: no per-chunk end-of-input checks
        const uint64_t full64 = c.len_in >> 16;
        const uint32_t nfull = (uint32_t)(full64 < grid.x ? full64 : grid.x);
        ContigArgs cc = c;
        if (nfull) FO_TRY(launch(pl, KID_ENC_PAIR, k_contig_pair<true, false, false>, dim3(nfull, grid.y), block, st, cc, tab));
        if (nfull < grid.x) {
            cc.tile0 = 2u * nfull;
            FO_TRY(launch(pl, KID_ENC_PAIR, k_contig_pair<true, false, true>, dim3(grid.x - nfull, grid.y), block, st, cc, tab));
        }
        return FO_OK;
    }
    return launch(pl, KID_ENC_PAIR, k_contig_pair<false, false>, grid, block, st, c, tab);
}

StridedArgs strided_base(const fo_plan *pl, const Rng &r, uint32_t pass)
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

ContigArgs contig_base(const fo_plan *pl, const Rng &r)
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
void set_quantiser(ContigArgs &c, const fo_plan *pl, uint32_t party)
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
uint32_t eps_party_of(const fo_plan *pl, uint32_t party)
{
    if (pl->p.eps_mode == FO_EPS_INDEPENDENT) return party;
    if (party == FO_PARTY_SERVER && pl->p.eps_mode == FO_EPS_SHARED_WORKERS) return party;
    return kPartyAllWorkers;
}

// Encode `nslots` vectors.  Sources: tab (pointer table, nslots entries) or src + slot * src_stride.
// scales_given: scales[] already holds the amplitudes (forced / bound rule); else they come from the
// measured norms.  common: the nslots parties are all the workers of a shared-eps round and must agree
// on one amplitude per block (the largest) before any of them quantises; scales is then [M][nblocks].
int launch_encode(fo_plan *pl, const PtrTab *tab, const float *src, uint64_t src_stride, uint64_t len_in,
                  uint32_t nslots, uint32_t party0, uint64_t round, bool scales_given, uint64_t *bits,
                  uint64_t bits_stride, float *scales, uint64_t scales_stride, float *tmp, uint64_t tmp_stride,
                  hipStream_t st, bool common = false)
{
    const Rng r = rng_of(pl, round);
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    const PtrTab &tb = tab ? *tab : none;
    const dim3 grid((unsigned)pl->ntiles, nslots), block(kThreads);
    ContigArgs c = contig_base(pl, r);
    c.dst = bits; c.dst_stride = bits_stride;
    c.scales = scales; c.scales_stride = scales_stride;
    c.party0 = party0; c.eps_party0 = eps_party_of(pl, party0);
    set_quantiser(c, pl, party0);
    // amplitude from a measured norm: alpha for a worker, alpha_s for the server's own vector
    const float coef = party0 == FO_PARTY_SERVER ? pl->coef_lambda_s : pl->coef_lambda;
    c.coef_lambda = coef;
    const dim3 cgrid((unsigned)((pl->nblocks + 255) / 256));
    if (pl->npass == 0) {
        c.src = src; c.src_stride = src_stride; c.use_tab = tab ? 1u : 0u;
        c.len_in = len_in;
        c.compute_scale = scales_given ? 0u : 1u;
        if (common && !scales_given) {
            // one extra read of the gradients: norms first, then the common amplitude, then the encode proper
            c.scales_only = 1u;
            FO_TRY(launch_pack<IN_GRAD>(pl, KID_ENC_SINGLE, grid, st, c, tb));
            FO_TRY(launch(pl, KID_SCALES, k_common_scales, cgrid, dim3(256), st, scales, pl->nblocks, nslots));
            c.scales_only = 0u;
            c.compute_scale = 0u;
        }
        FO_TRY(launch_pack<IN_GRAD>(pl, KID_ENC_SINGLE, grid, st, c, tb));
        return FO_OK;
    }
    if (pl->logb == 16 && !c.stat_clipped) {
        // blocks of exactly two tiles: one pass, a workgroup of 1024 threads per block
        c.src = src; c.src_stride = src_stride; c.use_tab = tab ? 1u : 0u;
        c.len_in = len_in;
        c.compute_scale = scales_given ? 0u : 1u;
        const dim3 pgrid((unsigned)(pl->ntiles / 2), nslots);
        if (common && !scales_given) {
            c.scales_only = 1u;
            FO_TRY(launch_pair(pl, pgrid, st, c, tb));
            FO_TRY(launch(pl, KID_SCALES, k_common_scales, cgrid, dim3(256), st, scales, pl->nblocks, nslots));
            c.scales_only = 0u;
            c.compute_scale = 0u;
        }
        return launch_pair(pl, pgrid, st, c, tb);
    }
    // transform lengths above 2^15: high stages first (eps flip and norm on load), low stages last
    const uint32_t first = pl->npass - 1;
    StridedArgs s = strided_base(pl, r, first);
    s.src = src; s.src_stride = src_stride; s.use_tab = tab ? 1u : 0u; s.len_in = len_in;
    s.dst = (pl->npass == 2) ? pl->buf_c : tmp; s.dst_stride = (pl->npass == 2) ? 0 : tmp_stride;
    s.partials = pl->partials; s.eps_party0 = eps_party_of(pl, party0);
    if (pl->npass == 2 && nslots != 1) return FO_EINVAL; // three-pass transforms are encoded one party at a time
    FO_TRY(launch_strided<SM_ENC_FIRST>(pl, KID_ENC_HIGH, grid, st, s, tb));
    if (pl->npass == 2) {
        StridedArgs s2 = strided_base(pl, r, 0);
        s2.src = pl->buf_c; s2.dst = tmp; s2.src_stride = 0; s2.dst_stride = tmp_stride;
        FO_TRY(launch_strided<SM_MID_F32>(pl, KID_ENC_MID, grid, st, s2, none));
    }
    if (!scales_given) {
        FO_TRY(launch(pl, KID_SCALES, k_finalize_scales, dim3((unsigned)pl->nblocks, nslots), dim3(256), st, pl->partials,
                           pl->ntiles, (uint32_t)(pl->b >> kTileLog2), coef, scales, scales_stride));
        if (common) FO_TRY(launch(pl, KID_SCALES, k_common_scales, cgrid, dim3(256), st, scales, pl->nblocks, nslots));
    }
    c.src = tmp; c.src_stride = tmp_stride;
    FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid, st, c, none));
    return FO_OK;
}

// Decode one party into out[len_out] with the given store mode.
int launch_decode(fo_plan *pl, const uint64_t *bits, const float *scales, uint64_t round, uint32_t party,
                  float *out, uint64_t len_out, uint32_t store_mode, float out_coef, float delta, float *tmp,
                  hipStream_t st)
{
    const Rng r = rng_of(pl, round);
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    const dim3 grid((unsigned)pl->ntiles, 1), block(kThreads);
    ContigArgs c = contig_base(pl, r);
    c.src = bits; c.src_stride = 0;
    c.scales = const_cast<float *>(scales); c.scales_stride = 0;
    c.party0 = party; c.eps_party0 = eps_party_of(pl, party);
    set_quantiser(c, pl, party);
    const bool multik = c.K > 1;
    // the decode-side transforms carry every value divided by two (see fo_contig.h); D = (lambda / K) D_eps H^T q
    out_coef *= 2.f / (float)c.K;
    if (pl->npass == 0) {
        c.dst = out; c.len_out = len_out; c.store_mode = store_mode; c.out_coef = out_coef; c.delta = delta;
        if (multik) FO_TRY(launch(pl, KID_DEC_SINGLE, (k_contig<IN_BITS, OUT_F32, false, false, 0, true>), grid, block, st, c, none));
        else if (c.S == 10) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<10>, grid, block, st, c));
        else if (c.S == 12) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<12>, grid, block, st, c));
        else if (c.S == 14) FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<14>, grid, block, st, c));
        else FO_TRY(launch(pl, KID_DEC_SINGLE, k_decode_tile<0>, grid, block, st, c));
        return FO_OK;
    }
    if (pl->logb == 16 && !multik) {
        // blocks of exactly two tiles: one pass, a workgroup of 1024 threads per block
        c.dst = out; c.len_out = len_out; c.store_mode = store_mode; c.out_coef = out_coef; c.delta = delta;
        return launch(pl, KID_DEC_PAIR, k_decode_pair, dim3((unsigned)(pl->ntiles / 2), 1), dim3(2 * kThreads), st, c);
    }
    c.dst = tmp; c.dst_stride = 0;
    StridedArgs s = strided_base(pl, r, pl->npass - 1);
    s.dst = out; s.len_out = len_out; s.store_mode = store_mode; s.out_coef = out_coef; s.delta = delta;
    s.scales = scales; s.scales_stride = 0; s.eps_party0 = eps_party_of(pl, party);
    if (pl->npass == 1 && !multik) {
        // int16 intermediate between the two passes
        FO_TRY(launch(pl, KID_DEC_LOW, k_declow, grid, block, st, c));
        s.src = tmp;
        FO_TRY((launch_strided<SM_DEC_LAST, true>(pl, KID_DEC_HIGH, grid, st, s, none)));
        return FO_OK;
    }
    if (multik) FO_TRY(launch(pl, KID_DEC_LOW, (k_contig<IN_BITS, OUT_I32, false, false, 15, true>), grid, block, st, c, none));
    else FO_TRY(launch(pl, KID_DEC_LOW, (k_contig<IN_BITS, OUT_I32, false, false, 15>), grid, block, st, c, none));
    if (pl->npass == 1) {
        s.src = tmp;
        FO_TRY(launch_strided<SM_DEC_LAST>(pl, KID_DEC_HIGH, grid, st, s, none));
        return FO_OK;
    }
    StridedArgs s1 = strided_base(pl, r, 0);
    s1.src = tmp; s1.dst = pl->buf_c;
    FO_TRY(launch_strided<SM_MID_I32>(pl, KID_DEC_MID, grid, st, s1, none));
    s.src = pl->buf_c;
    FO_TRY(launch_strided<SM_DEC_LAST>(pl, KID_DEC_HIGH, grid, st, s, none));
    return FO_OK;
}

int launch_server(fo_plan *pl, const uint64_t *bits_up, const float *scales_up, uint64_t round, uint64_t *bits_down,
                  float *scales_down, float *gbar_or_null, hipStream_t st)
{
    const Rng r = rng_of(pl, round);
    const uint32_t M = pl->p.M;
    PtrTab none;
    std::memset(&none, 0, sizeof(none));
    // server amplitude: the theorem's rule from the workers' amplitudes now, or from the norm of the mean later
    const bool l2s = pl->p.server_scale == FO_SERVER_SCALE_L2;
    if (!l2s)
        FO_TRY(launch(pl, KID_SCALES, k_server_scales, dim3((unsigned)((pl->nblocks + 255) / 256)), dim3(256), st, scales_up,
                           pl->nblocks, M, pl->coef_s, scales_down));
    auto finalize_server_scales = [&]() -> int { // after a fused strided pass that left the tile sums of squares of gbar
        return launch(pl, KID_SCALES, k_finalize_scales, dim3((unsigned)pl->nblocks, 1), dim3(256), st, pl->partials, pl->ntiles,
                      (uint32_t)(pl->b >> kTileLog2), pl->coef_lambda_s, scales_down, (uint64_t)0);
    };
    const float mean_coef = pl->rsqrtb / (float)M;
    const bool zero_transform = pl->p.eps_mode == FO_EPS_SHARED_ALL;
    if (zero_transform) {
        // the server shares the workers' eps: its pre-quantisation vector is (lambda / M)(2 c - M), no transform
        ShallArgs z;
        z.bits_up = bits_up; z.dst = bits_down; z.lam = scales_up; z.lam_s = scales_down;
        z.W = pl->W; z.logb = pl->logb; z.M = M; z.K = pl->p.K; z.planes = pl->planes; z.dither = pl->p.dither;
        z.k0 = r.k0; z.k1 = r.k1; z.round_lo = r.round_lo; z.round_dev = r.round_dev; z.sqrtb = pl->sqrtb;
        if (l2s) { // lambda^s from ||gbar||: an exact integer count first
            const dim3 bg((unsigned)((pl->nblocks + 255) / 256));
            FO_TRY(launch(pl, KID_SCALES, k_zero_u64, bg, dim3(256), st, pl->blk_sums, pl->nblocks));
            FO_TRY(launch(pl, KID_SHALL, k_shall_sumsq, dim3((unsigned)((pl->W + 15) / 16)), dim3(256), st, z, pl->blk_sums));
            FO_TRY(launch(pl, KID_SCALES, k_shall_scales, bg, dim3(256), st, pl->blk_sums, scales_up, pl->nblocks, M,
                          pl->coef_lambda_s, scales_down));
        }
        FO_TRY(launch(pl, KID_SHALL, k_shall, dim3((unsigned)((pl->W + 15) / 16)), dim3(256), st, z));
        if (!gbar_or_null) return FO_OK;
        // the mean itself was asked for (checking): one inverse transform of the summed sign vectors, below
    }
    if (pl->p.eps_mode != FO_EPS_INDEPENDENT && pl->npass <= 1) {
        // one eps and one amplitude for all workers: sum the packed sign vectors per coordinate (vertical
        // popcount), then a single inverse transform instead of M
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W; c.M = M;
        c.scales = const_cast<float *>(scales_up); c.scales_stride = 0; // worker 0's amplitudes are everybody's
        c.party0 = 0; c.eps_party0 = kPartyAllWorkers;
        const dim3 grid1((unsigned)pl->ntiles, 1), block(kThreads);
        if (pl->npass == 0) {
            float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
            c.dst = gbar; c.len_out = pl->ntot; c.store_mode = STORE_SET; c.out_coef = mean_coef;
            FO_TRY(launch(pl, KID_COUNT_LOW, (k_contig<IN_COUNT, OUT_F32>), grid1, block, st, c, none));
            if (zero_transform) return FO_OK;
            return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down,
                                 0, nullptr, 0, st);
        }
        c.dst = pl->buf_a; c.dst_stride = 0;
        FO_TRY(launch(pl, KID_COUNT_LOW, (k_contig<IN_COUNT, OUT_I32, false, false, 15>), grid1, block, st, c, none));
        StridedArgs s = strided_base(pl, r, 0);
        s.src = pl->buf_a; s.dst = pl->buf_b;
        s.scales = scales_up; s.scales_stride = 0;
        s.gbar = gbar_or_null;
        s.out_coef = mean_coef; s.eps_party0 = FO_PARTY_SERVER;
        s.partials = l2s ? pl->partials : nullptr;
        FO_TRY(launch_strided<SM_SHARED>(pl, KID_SERVER_HIGH, grid1, st, s, none));
        if (zero_transform) return FO_OK;
        if (l2s) FO_TRY(finalize_server_scales());
        ContigArgs e = contig_base(pl, r);
        e.src = pl->buf_b; e.dst = bits_down;
        e.scales = scales_down;
        e.party0 = FO_PARTY_SERVER; e.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(e, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, grid1, st, e, none));
        return FO_OK;
    }
    if (pl->npass == 0) {
        // the transform fits a tile: the mean tile by tile in registers, then the ordinary encode
        float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
        ServerTileArgs sa;
        sa.enc = contig_base(pl, r);
        sa.enc.src = gbar;
        sa.bits_up = bits_up; sa.scales_up = scales_up; sa.M = M;
        sa.coef = 2.f * mean_coef; // the decode side carries half values
        const dim3 mgrid((unsigned)pl->ntiles, 1), mblock(kThreads);
        if (pl->S == 10) FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_tile<10>, mgrid, mblock, st, sa));
        else if (pl->S == 12) FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_tile<12>, mgrid, mblock, st, sa));
        else if (pl->S == 14) FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_tile<14>, mgrid, mblock, st, sa));
        else FO_TRY(launch(pl, KID_SERVER_TILE, k_mean_tile<0>, mgrid, mblock, st, sa));
        return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down, 0,
                             nullptr, 0, st);
    }
    if (pl->npass == 2) {
        // three-pass transforms: unfused (decode each worker into the mean, then a plain encode)
        float *gbar = gbar_or_null ? gbar_or_null : pl->buf_b;
        for (uint32_t m = 0; m < M; ++m) {
            int rc = launch_decode(pl, bits_up + (uint64_t)m * pl->W, scales_up + (uint64_t)m * pl->nblocks, round, m, gbar,
                                   pl->ntot, m == 0 ? STORE_SET : STORE_ACC, mean_coef, 0.f, pl->buf_a, st);
            if (rc) return rc;
        }
        return launch_encode(pl, nullptr, gbar, 0, pl->ntot, 1, FO_PARTY_SERVER, round, !l2s, bits_down, 0, scales_down, 0,
                             pl->buf_a, 0, st);
    }
    // two-pass transforms: M low-stage passes (bits -> int32), one fused high-stage pass that forms the mean
    // and starts the re-encode, one low-stage pass that dithers and packs
    {
        ContigArgs c = contig_base(pl, r);
        c.src = bits_up; c.src_stride = pl->W;
        c.dst = pl->buf_a; c.dst_stride = pl->ntot;
        FO_TRY(launch(pl, KID_DEC_LOW, k_declow, dim3((unsigned)pl->ntiles, M), dim3(kThreads), st, c));
    }
    {
        StridedArgs s = strided_base(pl, r, 0);
        s.src = pl->buf_a; s.src_stride = pl->ntot;
        s.dst = pl->buf_b;
        s.scales = scales_up; s.scales_stride = pl->nblocks;
        s.gbar = gbar_or_null;
        s.M = M; s.out_coef = 2.f * mean_coef; s.eps_party0 = FO_PARTY_SERVER; // int16 input holds half values
        s.partials = l2s ? pl->partials : nullptr;
        FO_TRY((launch_strided<SM_SERVER, true>(pl, KID_SERVER_HIGH, dim3((unsigned)pl->ntiles, 1), st, s, none)));
        if (l2s) FO_TRY(finalize_server_scales());
    }
    {
        ContigArgs c = contig_base(pl, r);
        c.src = pl->buf_b; c.src_stride = 0;
        c.dst = bits_down; c.dst_stride = 0;
        c.scales = scales_down; c.scales_stride = 0;
        c.party0 = FO_PARTY_SERVER; c.eps_party0 = FO_PARTY_SERVER;
        set_quantiser(c, pl, FO_PARTY_SERVER);
        FO_TRY(launch_pack<IN_F32>(pl, KID_ENC_LOW, dim3((unsigned)pl->ntiles, 1), st, c, none));
    }
    return FO_OK;
}

int prepare_scales(fo_plan *pl, uint32_t nslots, bool forced, float *scales, uint64_t scales_stride, hipStream_t st,
                   bool *given)
{
    *given = forced;
    if (!forced && pl->p.scale_rule == FO_SCALE_BOUND) {
        FO_TRY(launch(pl, KID_SCALES, k_fill_scales, dim3((unsigned)((pl->nblocks + 255) / 256), nslots), dim3(256), st, scales,
                           scales_stride, pl->nblocks, pl->coef_lambda * pl->p.B));
        *given = true;
    }
    return FO_OK;
}

} // namespace

extern "C" int fo_encode(fo_plan *pl, const float *g, uint64_t round, uint32_t party, uint32_t flags, uint64_t *bits,
                         float *scales, void *hip_stream)
{
    if (!pl || !g || !bits || !scales) return FO_EINVAL;
    if (party != FO_PARTY_SERVER && party >= pl->p.M) return FO_EINVAL;
    if (flags & ~FO_FORCE_SCALE) return FO_EINVAL;
    if (!aligned(g, 16) || !aligned(bits, 8) || !aligned(scales, 4)) return FO_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    bool given;
    int rc = prepare_scales(pl, 1, (flags & FO_FORCE_SCALE) != 0, scales, 0, st, &given);
    if (rc) return rc;
    const uint64_t len = party == FO_PARTY_SERVER ? pl->ntot : pl->p.d;
    return launch_encode(pl, nullptr, g, 0, len, 1, party, round, given, bits, 0, scales, 0, pl->buf_a, 0, st);
}

extern "C" int fo_decode(fo_plan *pl, const uint64_t *bits, const float *scales, uint64_t round, uint32_t party,
                         float *out, void *hip_stream)
{
    if (!pl || !bits || !scales || !out) return FO_EINVAL;
    if (party != FO_PARTY_SERVER && party >= pl->p.M) return FO_EINVAL;
    if (!aligned(bits, 8) || !aligned(scales, 4) || !aligned(out, 16)) return FO_EALIGN;
    return launch_decode(pl, bits, scales, round, party, out, pl->p.d, STORE_SET, pl->rsqrtb, 0.f, pl->buf_a,
                         static_cast<hipStream_t>(hip_stream));
}

extern "C" int fo_server_aggregate(fo_plan *pl, const uint64_t *bits_up, const float *scales_up, uint64_t round,
                                   uint64_t *bits_down, float *scales_down, float *gbar_or_null, void *hip_stream)
{
    if (!pl || !bits_up || !scales_up || !bits_down || !scales_down) return FO_EINVAL;
    if (!aligned(bits_up, 8) || !aligned(scales_up, 4) || !aligned(bits_down, 8) || !aligned(scales_down, 4) ||
        !aligned(gbar_or_null, 16))
        return FO_EALIGN;
    return launch_server(pl, bits_up, scales_up, round, bits_down, scales_down, gbar_or_null,
                         static_cast<hipStream_t>(hip_stream));
}

extern "C" int fo_step(fo_plan *pl, const float *const *g, float *x, float delta, uint64_t round, void *hip_stream)
{
    if (!pl || !g || !x) return FO_EINVAL;
    if (!aligned(x, 16)) return FO_EALIGN;
    PtrTab tab;
    std::memset(&tab, 0, sizeof(tab));
    for (uint32_t m = 0; m < pl->p.M; ++m) {
        if (!g[m]) return FO_EINVAL;
        if (!aligned(g[m], 16)) return FO_EALIGN;
        tab.p[m] = g[m];
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const uint32_t M = pl->p.M;
    bool given;
    int rc = prepare_scales(pl, M, false, pl->scales_up, pl->nblocks, st, &given);
    if (rc) return rc;
    if (pl->npass == 2) {
        for (uint32_t m = 0; m < M && !rc; ++m)
            rc = launch_encode(pl, nullptr, g[m], 0, pl->p.d, 1, m, round, given, pl->bits_up + (uint64_t)m * pl->W, 0,
                               pl->scales_up + (uint64_t)m * pl->nblocks, 0, pl->buf_a, 0, st);
    } else {
        rc = launch_encode(pl, &tab, nullptr, 0, pl->p.d, M, 0, round, given, pl->bits_up, pl->W, pl->scales_up,
                           pl->nblocks, pl->buf_a, pl->ntot, st, pl->p.eps_mode != FO_EPS_INDEPENDENT);
    }
    if (rc) return rc;
    rc = launch_server(pl, pl->bits_up, pl->scales_up, round, pl->bits_down, pl->scales_down, nullptr, st);
    if (rc) return rc;
    return launch_decode(pl, pl->bits_down, pl->scales_down, round, FO_PARTY_SERVER, x, pl->p.d, STORE_AXPY, pl->rsqrtb,
                         delta, pl->buf_a, st);
}

extern "C" int fo_step_dev_round(fo_plan *pl, const float *const *g, float *x, float delta, const uint64_t *round_dev,
                                 void *hip_stream)
{
    if (!pl || !round_dev) return FO_EINVAL;
    if (!aligned(round_dev, 8)) return FO_EALIGN;
    pl->round_dev = reinterpret_cast<const unsigned long long *>(round_dev);
    const int rc = fo_step(pl, g, x, delta, 0, hip_stream);
    pl->round_dev = nullptr;
    return rc;
}

extern "C" int fo_set_stats(fo_plan *pl, fo_stats *stats)
{
    if (!pl) return FO_EINVAL;
    if (!aligned(stats, 8)) return FO_EALIGN;
    pl->stats = stats;
    return FO_OK;
}

extern "C" int fo_step_messages(fo_plan *pl, const uint64_t **bits_up, const float **scales_up,
                                const uint64_t **bits_down, const float **scales_down)
{
    if (!pl) return FO_EINVAL;
    if (bits_up) *bits_up = pl->bits_up;
    if (scales_up) *scales_up = pl->scales_up;
    if (bits_down) *bits_down = pl->bits_down;
    if (scales_down) *scales_down = pl->scales_down;
    return FO_OK;
}

extern "C" int fo_profile_begin(fo_plan *pl)
{
    if (!pl) return FO_EINVAL;
    Profiler &pf = pl->prof;
    if (!pf.ev) {
        pf.ev = new (std::nothrow) hipEvent_t[2 * Profiler::kMax];
        pf.kid = new (std::nothrow) int[Profiler::kMax];
        if (!pf.ev || !pf.kid) return FO_ENOMEM;
        for (int i = 0; i < 2 * Profiler::kMax; ++i)
            if (!hip_ok(hipEventCreate(&pf.ev[i]), "hipEventCreate")) return FO_EHIP;
    }
    pf.used = 0;
    pf.only = -1;
    pf.on = true;
    return FO_OK;
}

extern "C" int fo_profile_begin_kernel(fo_plan *pl, const char *kernel_name)
{
    if (!pl || !kernel_name) return FO_EINVAL;
    int kid = -1;
    for (int k = 0; k < KID_COUNT; ++k)
        if (std::strcmp(kKernelNames[k], kernel_name) == 0) kid = k;
    if (kid < 0) return FO_EINVAL;
    const int rc = fo_profile_begin(pl);
    if (rc) return rc;
    pl->prof.only = kid;
    return FO_OK;
}

extern "C" int fo_profile_end(fo_plan *pl, fo_kernel_time *out, size_t cap, size_t *count)
{
    if (!pl || !out || !count) return FO_EINVAL;
    Profiler &pf = pl->prof;
    if (!pf.on) return FO_EINVAL;
    pf.on = false;
    float total[KID_COUNT] = { 0 };
    uint32_t launches[KID_COUNT] = { 0 };
    for (int i = 0; i < pf.used; ++i) {
        if (!hip_ok(hipEventSynchronize(pf.ev[2 * i + 1]), "hipEventSynchronize")) return FO_EHIP;
        float ms = 0.f;
        if (!hip_ok(hipEventElapsedTime(&ms, pf.ev[2 * i], pf.ev[2 * i + 1]), "hipEventElapsedTime")) return FO_EHIP;
        total[pf.kid[i]] += ms;
        launches[pf.kid[i]] += 1;
    }
    size_t n = 0;
    for (int k = 0; k < KID_COUNT && n < cap; ++k) {
        if (!launches[k]) continue;
        std::snprintf(out[n].name, sizeof(out[n].name), "%s", kKernelNames[k]);
        out[n].launches = launches[k];
        out[n].total_ms = total[k];
        ++n;
    }
    *count = n;
    return FO_OK;
}

// ---------------------------------------------------------------------------------------------
// Encode without any allocation: intermediates in a static device array
// ---------------------------------------------------------------------------------------------
namespace {

constexpr uint64_t kNoallocMaxN = (uint64_t)FO_NOALLOC_MAX_N;
constexpr uint64_t kNoallocPartials = kNoallocMaxN >> kTileLog2;          // one sum of squares per tile
constexpr uint64_t kNoallocWords = kNoallocMaxN + ((kNoallocPartials + 63) & ~(uint64_t)63);

} // namespace

// fp32 intermediate of the two-pass encode [FO_NOALLOC_MAX_N], then the tile sums of squares.  Every device the
// library runs on holds its own copy until the process ends.  Host code never uses this name as an address: the
// per-device address comes from hipGetSymbolAddress (noalloc_scratch below).
static __device__ __align__(256) float scratch[kNoallocWords];

namespace {

constexpr int kMaxDevices = 64;
float *g_scratch_ptr[kMaxDevices]; // device address of `scratch` on each device, set by the first call there

int noalloc_scratch(float **out)
{
    int dev = -1;
    if (!hip_ok(hipGetDevice(&dev), "hipGetDevice")) return FO_EHIP;
    if (dev < 0 || dev >= kMaxDevices) {
        std::snprintf(g_hip_err, sizeof(g_hip_err), "fo_encode_noalloc: device ordinal %d not supported", dev);
        return FO_EHIP;
    }
    float *p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        void *sym = nullptr;
        if (!hip_ok(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)")) return FO_EHIP;
        if (!sym) {
            std::snprintf(g_hip_err, sizeof(g_hip_err), "fo_encode_noalloc: no address for the static scratch array");
            return FO_EHIP;
        }
        p = static_cast<float *>(sym);
        __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE); // every thread would store the same value
    }
    *out = p;
    return FO_OK;
}

} // namespace

extern "C" int fo_encode_noalloc(const fo_params *params, const float *g, uint64_t round, uint32_t party, uint32_t flags,
                                 uint64_t *bits, float *scales, void *hip_stream)
{
    if (!params || !g || !bits || !scales) return FO_EINVAL;
    fo_plan pl; // host object on the stack: geometry only, no device memory of its own
    {
        const int rc = plan_geometry(*params, &pl);
        if (rc) return rc;
    }
    if (pl.ntot > kNoallocMaxN) {
        std::snprintf(g_hip_err, sizeof(g_hip_err), "fo_encode_noalloc: padded length %llu exceeds FO_NOALLOC_MAX_N = %llu",
                      (unsigned long long)pl.ntot, (unsigned long long)kNoallocMaxN);
        return FO_ESIZE;
    }
    if (party != FO_PARTY_SERVER && party >= pl.p.M) return FO_EINVAL;
    if (flags & ~FO_FORCE_SCALE) return FO_EINVAL;
    if (!aligned(g, 16) || !aligned(bits, 8) || !aligned(scales, 4)) return FO_EALIGN;
    float *ptr = nullptr;
    {
        const int rc = noalloc_scratch(&ptr);
        if (rc) return rc;
    }
    pl.scratch = nullptr;
    pl.scratch_bytes = 0;
    pl.buf_a = ptr;                 // fp32 intermediate between the strided and the contiguous pass
    pl.buf_b = pl.buf_c = nullptr;  // transforms of up to 2^22 points never take a third pass
    pl.partials = ptr + kNoallocMaxN;
    pl.bits_up = pl.bits_down = nullptr;
    pl.scales_up = pl.scales_down = nullptr;
    pl.blk_sums = nullptr;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    bool given;
    int rc = prepare_scales(&pl, 1, (flags & FO_FORCE_SCALE) != 0, scales, 0, st, &given);
    if (rc) return rc;
    const uint64_t len = party == FO_PARTY_SERVER ? pl.ntot : pl.p.d;
    return launch_encode(&pl, nullptr, g, 0, len, 1, party, round, given, bits, 0, scales, 0, pl.buf_a, 0, st);
}
