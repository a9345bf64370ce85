// C ABI of the FO-SGD codec (declared in include/fo.h): argument checks, plan scratch and the small amplitude
// kernels.  The launch sequences live in fo_enc.hip, fo_dec.hip and fo_srv.hip.
#include <cstdlib>
#include "fo_host.h"

using namespace fo;
using namespace fo_host;

namespace fo_host {
thread_local char g_hip_err[256] = "";
}

namespace {

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

} // namespace

namespace fo_host {

int launch_finalize_scales(fo_plan *pl, hipStream_t st, uint32_t nslots, float coef, float *scales, uint64_t scales_stride)
{
    return launch(pl, KID_SCALES, k_finalize_scales, dim3((unsigned)pl->nblocks, nslots), dim3(256), st, pl->partials, pl->ntiles,
                  (uint32_t)(pl->b >> kTileLog2), coef, scales, scales_stride);
}
int launch_fill_scales(fo_plan *pl, hipStream_t st, uint32_t nslots, float *scales, uint64_t scales_stride, float value)
{
    return launch(pl, KID_SCALES, k_fill_scales, dim3((unsigned)((pl->nblocks + 255) / 256), nslots), dim3(256), st, scales,
                  scales_stride, pl->nblocks, value);
}
int launch_server_scales(fo_plan *pl, hipStream_t st, const float *scales_up, float *scales_down)
{
    return launch(pl, KID_SCALES, k_server_scales, dim3((unsigned)((pl->nblocks + 255) / 256)), dim3(256), st, scales_up,
                  pl->nblocks, pl->p.M, pl->coef_s, scales_down);
}
int launch_common_scales(fo_plan *pl, hipStream_t st, float *scales, uint32_t nslots)
{
    return launch(pl, KID_SCALES, k_common_scales, dim3((unsigned)((pl->nblocks + 255) / 256)), dim3(256), st, scales,
                  pl->nblocks, nslots);
}

} // namespace fo_host

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
    if (q.server_scale != FO_SERVER_SCALE_THM && q.server_scale != FO_SERVER_SCALE_L2 && q.server_scale != FO_SERVER_SCALE_SUP)
        return FO_EINVAL;
    // lambda^s = lambda is admissible only where the server's vector is bounded by lambda surely
    if (q.server_scale == FO_SERVER_SCALE_SUP && q.eps_mode != FO_EPS_SHARED_ALL) return FO_EINVAL;

    pl->p = q;
    pl->stats = nullptr;
    pl->round_dev = nullptr;
    pl->num_cus = 256;
    pl->pad32 = pl->pad16 = 0;
    // FO_SERVER_VECTOR_UNIT=1 in the environment keeps the server pass of 2^25-blocks on the vector-unit kernel: the two
    // kernels give the same bits, and the tests use the switch to show it
    {
        const char *e = std::getenv("FO_SERVER_VECTOR_UNIT");
        pl->server_mfma = !(e && e[0] == '1');
    }
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
    // shared eps: the sum of the M sign vectors is transformed in int32, magnitudes up to M b
    if (q.eps_mode != FO_EPS_INDEPENDENT && (uint64_t)q.M * pl->b >= ((uint64_t)1 << 31)) return FO_EINVAL;
    pl->planes = 0;
    while ((q.K >> pl->planes) != 0) ++pl->planes;
    // the decode side carries K b / 2 at most in int32 between its passes
    if (q.K > 1 && pl->npass > 0 && (uint64_t)q.K * (pl->b / 2) >= ((uint64_t)1 << 31)) return FO_EINVAL;
    const double bd = (double)pl->b;
    pl->coef_lambda = (float)((double)q.alpha * std::sqrt(std::log(bd) / bd));
    pl->sqrtb = (float)std::sqrt(bd);
    pl->rsqrtb = (float)(1.0 / std::sqrt(bd));
    pl->coef_s = q.server_scale == FO_SERVER_SCALE_SUP ? 1.f : (float)((double)q.alpha_s * std::sqrt(std::log(bd)));
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

    {
        int dev = 0, cus = 0;
        if (!hip_ok(hipGetDevice(&dev), "hipGetDevice") ||
            !hip_ok(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev), "hipDeviceGetAttribute")) {
            delete pl;
            return FO_EHIP;
        }
        if (cus > 0) pl->num_cus = (uint32_t)cus;
    }
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    if (pl->npass == 1) { pl->pad32 = kRowPad32; pl->pad16 = kRowPad16; }
    const size_t sz_a = pl->npass ? up((size_t)q.M * (pl->ntot + pl->ntiles * pl->pad32) * 4) : 0;
    const size_t sz_b = up((pl->ntot + pl->ntiles * pl->pad32) * 4);
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

namespace {

int prepare_scales(fo_plan *pl, uint32_t nslots, bool forced, float *scales, uint64_t scales_stride, hipStream_t st,
                   bool *given)
{
    *given = forced;
    if (!forced && pl->p.scale_rule == FO_SCALE_BOUND) {
        FO_TRY(launch_fill_scales(pl, st, nslots, scales, scales_stride, pl->coef_lambda * pl->p.B));
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
        // three-pass transforms are encoded one worker at a time.  With a shared eps the workers must agree on one
        // amplitude per block before any of them quantises: a first round of encodes only measures the norms (its
        // messages are overwritten by the second), then the largest amplitude is everybody's.
        if (pl->p.eps_mode != FO_EPS_INDEPENDENT && !given) {
            for (uint32_t m = 0; m < M && !rc; ++m)
                rc = launch_encode(pl, nullptr, g[m], 0, pl->p.d, 1, m, round, false, pl->bits_up + (uint64_t)m * pl->W, 0,
                                   pl->scales_up + (uint64_t)m * pl->nblocks, 0, pl->buf_a, 0, st);
            if (rc) return rc;
            rc = launch_common_scales(pl, st, pl->scales_up, M);
            if (rc) return rc;
            given = true;
        }
        for (uint32_t m = 0; m < M && !rc; ++m)
            rc = launch_encode(pl, nullptr, g[m], 0, pl->p.d, 1, m, round, given, pl->bits_up + (uint64_t)m * pl->W, 0,
                               pl->scales_up + (uint64_t)m * pl->nblocks, 0, pl->buf_a, 0, st);
    } else {
        rc = launch_encode(pl, &tab, nullptr, 0, pl->p.d, M, 0, round, given, pl->bits_up, pl->W, pl->scales_up,
                           pl->nblocks, pl->buf_a, pl->ntot + pl->ntiles * pl->pad32, st, pl->p.eps_mode != FO_EPS_INDEPENDENT);
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

