/*
 * fo.h -- C ABI of the MI355X (gfx950) FO-SGD gradient codec.
 *
 * Paper: "Flattened one-bit stochastic gradient descent", arXiv 2405.11095.  One FO-SGD
 * iteration (Sec. 4) is: every worker n encodes its gradient g_n with the (eps_n, lambda)-encoder
 * of Def. 3.7 and sends d sign bits; the server decodes each message with the decoder of
 * Def. 3.8, averages (eq. "server average"), re-encodes the mean with the
 * (eps^s, lambda^s, K)-encoder and sends it down; every worker decodes it and takes the step
 * x <- x - delta * g^d.  This library is that codec.  The M workers are M buffers on one device.
 *
 * Conventions common to all calls
 *   - Every pointer named "device" is a device (HBM) pointer owned by the caller.  The library
 *     never frees or keeps them beyond the call's enqueued work.  Alignment (FO_EALIGN otherwise):
 *     fp32 vectors (g, gbar, out, x) 16 bytes, packed words 8 bytes, scales 4 bytes.  Host
 *     pointers are said to be host.
 *   - All work is enqueued on the caller's HIP stream (a hipStream_t passed as void*; NULL is the
 *     default stream).  The hot calls (fo_encode, fo_decode, fo_server_aggregate, fo_step) do
 *     not allocate, do not synchronise with the host and copy nothing between host and device;
 *     scratch memory is allocated once by fo_plan_create.
 *   - Return value: 0 (FO_OK) or a negative FO_E* code.  No exception crosses the boundary.
 *   - A plan is not thread-safe; calls on one plan must not overlap on the device.
 *   - Output buffers must not alias inputs (x in fo_step is updated in place by design).
 *
 * Geometry.  With block_log2 = 0 the transform length is n = max(64, 2^ceil(log2 d)) and the
 * gradient is zero-padded to n (the paper assumes d a power of two, Def. 3.4).  With
 * block_log2 = k the gradient is cut into ceil(d / 2^k) blocks of b = 2^k coordinates (the last
 * zero-padded), each with its own transform and its own dither amplitude; the paper has no
 * blocked variant, Lemma A.7 with gamma = 1/sqrt(b) is what covers it.  Padded length
 * ntot = b * nblocks, packed words W = ntot / 64, scales per party = nblocks.
 *
 * Packed signs: word w, bit j  <->  coordinate 64 w + j; a set bit is +1.  sign(0) = +1.
 *
 * Scales.  A party's scales[j] is the dither amplitude lambda_j of block j in the paper's
 * (orthonormal) normalisation: lambda = alpha * B * sqrt(ln b / b) (Thm 5.5), with B the caller's
 * bound (FO_SCALE_BOUND) or the block's measured l2 norm (FO_SCALE_L2).  The server amplitude is
 * lambda^s_j = alpha_s * max_n lambda_{n,j} * sqrt(ln b) (Thm 5.5).  That rule bounds the mean by
 * ||gbar|| <= lambda sqrt(b); the server lemma in the proof only needs
 * lambda^s >= alpha_s sqrt(ln b / b) ||gbar||, and FO_SERVER_SCALE_L2 takes exactly that, with the norm of
 * the mean the server has just formed.  It is between sqrt(M) (when the uplink's quantisation noise dominates
 * gbar, the usual case) and alpha sqrt(ln b) times smaller, which cuts the downlink's error term by that
 * factor squared.  With FO_EPS_SHARED_ALL the vector the server quantises is (lambda / M)(2 c - M), bounded by
 * lambda in every coordinate for every eps, and the quantiser of Def. 3.2 is unbiased whenever the sup norm of its
 * input is at most its amplitude: FO_SERVER_SCALE_SUP then takes lambda^s = lambda, the workers' common amplitude,
 * alpha_s sqrt(ln b) times below the theorem's rule (other eps modes reject it with FO_EINVAL).
 *
 * Amplitudes a caller supplies (FO_FORCE_SCALE, fo_decode, fo_server_aggregate) may have either sign: the decoder is
 * linear in them, so a negated amplitude gives the negated vector on every path.
 *
 * Shared worker eps (FO_EPS_SHARED_WORKERS, a variant the paper does not have).  When every worker
 * uses the same eps_t and the same amplitude, linearity of H^T turns the server's M decodes into one:
 * gbar = (lambda / M) D_eps H^T (2 c - M) with c the per-coordinate count of set bits over the M
 * messages (a vertical popcount).  The server eps stays independent, as the server lemma in the proof
 * of Thm 5.5 needs.  fo_step agrees on the common amplitude by itself (per block, the largest of the
 * workers' amplitudes); a caller driving fo_encode by hand must pass that amplitude with
 * FO_FORCE_SCALE, and fo_server_aggregate then reads worker 0's scales as everybody's.
 *
 * FO_EPS_SHARED_ALL goes one step further and lets the server use the workers' eps too: then
 * H D_eps gbar = (lambda / M)(2 c - M) and the server needs no transform at all, only the count, the dither
 * and the comparison.  This drops the independence of eps^s that the paper's server lemma assumes; it is a
 * flagged variant, never the default.  gbar_or_null still works (one inverse transform, for checking).
 * Both shared modes need M b < 2^31 (the summed sign vectors are transformed in 32-bit integers).  For transform
 * lengths above 2^25 (three passes) fo_step measures the workers' norms in a first round of encodes before the
 * common amplitude is known, i.e. it encodes twice.
 *
 * Averaged downlink quantiser (K > 1).  The server's message is Q_{lambda^s,K} of Def. 3.2: the mean of K
 * one-bit quantisers with independent dithers, which cuts the downlink's error term by K (Lemma "Second
 * moment of the quantizer").  Coordinate i then carries the count c_i in {0..K} of dithers for which
 * sign(z_i + tau_{k,i}) = +1, so (K / lambda^s) Q_{lambda^s,K}(z)_i = 2 c_i - K, stored as
 * P = ceil(log2(K + 1)) bit planes of W words each (the paper's "log2(K+1) d bits"): plane p, word w,
 * bit j  <->  bit p of c_{64 w + j}.  Every downlink buffer (bits_down; bits of party FO_PARTY_SERVER) is
 * uint64[P][W]; fo_downlink_planes gives P.  Workers' messages always have K = 1 (Sec. 4).  K = 1 is the
 * plain sign message, P = 1.  Limit: K <= FO_MAX_K and, for transforms longer than 2^15, K * b < 2^32.
 *
 * Random numbers.  eps and the dither are functions of (seed, round, party, coordinate) through
 * Philox4x32-10; eps is therefore never transmitted, both ends regenerate it (the paper sends it
 * explicitly, Sec. 4 "Transmission").  The dither is u * lambda with u an odd multiple of 2^-24
 * in (-1, 1).
 */
#ifndef FO_H
#define FO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FO_OK 0
#define FO_EINVAL (-1) /* NULL / out-of-range argument, unsupported parameter value */
#define FO_EALIGN (-2) /* a device pointer is not aligned as required                      */
#define FO_EHIP (-3)   /* a HIP runtime call failed; see fo_last_hip_error              */
#define FO_ENOMEM (-4) /* plan creation could not allocate its scratch memory         */
#define FO_ESIZE (-5)  /* fo_encode_noalloc: vector longer than its static scratch takes  */

#define FO_DITHER_UNIFORM 0u /* tau ~ U[-lambda, lambda], Def. 3.2                       */
#define FO_DITHER_NONE 1u    /* tau = 0: plain sign of the flattened vector (ablation)   */
#define FO_SCALE_BOUND 0u    /* B is the caller's bound on ||g||_2 (Thm 5.5 verbatim)    */
#define FO_SCALE_L2 1u       /* B := measured ||g_block||_2 at this call                 */
#define FO_EPS_INDEPENDENT 0u /* one eps per worker and one for the server (Sec. 4)     */
#define FO_EPS_SHARED_WORKERS 1u /* one eps for all workers, an independent one for the server */
#define FO_EPS_SHARED_ALL 2u /* one eps for the workers and the server (flagged variant, see above) */

#define FO_SERVER_SCALE_THM 0u /* lambda^s = alpha_s max_n lambda_n sqrt(ln b)  (Thm 5.5 as stated)            */
#define FO_SERVER_SCALE_L2 1u  /* lambda^s = alpha_s sqrt(ln b / b) ||gbar_block||_2 (measured, see "Scales")  */
#define FO_SERVER_SCALE_SUP 2u /* lambda^s = max_n lambda_n; FO_EPS_SHARED_ALL only (see "Scales")              */

#define FO_PARTY_SERVER 0xFFFFFFFFu /* party id of the server; workers are 0 .. M-1      */
#define FO_FORCE_SCALE 1u /* fo_encode flag: scales[] is an input (amplitudes to use)    */

#define FO_MAX_WORKERS 64u
#define FO_NOALLOC_MAX_N (1u << 22) /* largest padded length fo_encode_noalloc takes */
#define FO_MAX_K 255u

typedef struct {
    uint64_t d;          /* logical gradient length, 1 <= d; one transform: d <= 2^30; blocked: ntot <= 2^32 */
    uint32_t M;          /* number of workers (the paper's N), 1 .. FO_MAX_WORKERS        */
    uint32_t block_log2; /* 0, or 6 .. 30                                                 */
    uint32_t K;          /* averaging count of the downlink quantizer (Def. 3.2), 1 .. FO_MAX_K */
    uint32_t dither;     /* FO_DITHER_*                                                   */
    uint32_t scale_rule; /* FO_SCALE_*                                                    */
    uint32_t eps_mode;   /* FO_EPS_*                                                      */
    float alpha;         /* worker amplitude factor, >= 2 (Lemma 3.6)                     */
    float alpha_s;       /* server amplitude factor, >= 2                                 */
    float B;             /* norm bound for FO_SCALE_BOUND, > 0 (ignored by FO_SCALE_L2)   */
    uint64_t seed;
    uint32_t server_scale; /* FO_SERVER_SCALE_*; 0 = the theorem's rule                        */
} fo_params;

typedef struct fo_plan fo_plan;

/* Validates *params (host), copies it and allocates the plan's device scratch on the current
 * device.  *out receives the plan (host object).  FO_EINVAL / FO_ENOMEM / FO_EHIP on failure. */
int fo_plan_create(const fo_params *params, fo_plan **out);
/* Frees the plan and its scratch.  The caller must have synchronised the streams it used. */
void fo_plan_destroy(fo_plan *plan);

size_t fo_padded_len(const fo_plan *plan);   /* ntot                                       */
size_t fo_packed_words(const fo_plan *plan); /* W = ntot / 64                              */
size_t fo_num_scales(const fo_plan *plan);   /* nblocks                                    */
size_t fo_block_len(const fo_plan *plan);    /* b                                          */
size_t fo_downlink_planes(const fo_plan *plan); /* P = ceil(log2(K + 1)) bit planes of a server message */
size_t fo_scratch_bytes(const fo_plan *plan);
/* Text of the last HIP error seen by this library on the calling thread (host string). */
const char *fo_last_hip_error(void);

/* Encoder E_{eps,lambda}(g) = sign(H D_eps g + tau), Def. 3.7 (Sec. 4, "Encoding"); K = 1 for a worker,
 * the plan's K for party FO_PARTY_SERVER (then bits is uint64[P][W], see "Averaged downlink quantiser").
 *   g       device fp32[len]: len = d for a worker, ntot when party == FO_PARTY_SERVER
 *   round   iteration t; party: worker id < M, or FO_PARTY_SERVER
 *   flags   0: scales[] is written with the amplitudes the rule gives (a worker: alpha and the plan's scale
 *           rule.  Party FO_PARTY_SERVER on its own knows no worker amplitudes, so Thm 5.5's server rule is
 *           left to fo_server_aggregate; here it gets alpha_s sqrt(ln b / b) ||g_block|| under FO_SCALE_L2
 *           and alpha B sqrt(ln b / b) under FO_SCALE_BOUND);
 *           FO_FORCE_SCALE: scales[] is read and used as given
 *   bits    device uint64[W] out;  scales device fp32[nblocks] in or out                      */
int fo_encode(fo_plan *plan, const float *g, uint64_t round, uint32_t party, uint32_t flags,
              uint64_t *bits, float *scales, void *hip_stream);

/* Decoder D_{eps,lambda,K}(q) = (lambda / K) D_eps H^T q, Def. 3.8 (Sec. 4, "Decoding"); K = 1 for a worker's
 * message, the plan's K for party FO_PARTY_SERVER.
 *   bits device uint64[W] (uint64[P][W] for the server's message), scales device fp32[nblocks] (as produced
 *   by the matching encode)
 *   out  device fp32[d]: the first d coordinates of the decoded vector                          */
int fo_decode(fo_plan *plan, const uint64_t *bits, const float *scales, uint64_t round,
              uint32_t party, float *out, void *hip_stream);

/* Server: gbar = (1/M) sum_n D_{eps_n,lambda_n}(q_n) (eq. "server average"), then the
 * (eps^s, lambda^s)-encoder applied to gbar in R^ntot (Sec. 4, "Server-to-workers").
 *   bits_up     device uint64[M][W];   scales_up   device fp32[M][nblocks]
 *   bits_down   device uint64[P][W] out (P = 1 when K = 1);  scales_down device fp32[nblocks] out (lambda^s)
 *   gbar_or_null  optional device fp32[ntot] out: the mean, materialised (for checking)         */
int fo_server_aggregate(fo_plan *plan, const uint64_t *bits_up, const float *scales_up,
                        uint64_t round, uint64_t *bits_down, float *scales_down,
                        float *gbar_or_null, void *hip_stream);

/* fo_encode for callers that cannot allocate device memory: code running under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  No plan: the geometry is derived from *params (host) at every call,
 * and the intermediates of transforms longer than 2^15 points (an fp32 vector of the padded length and one sum
 * of squares per tile) live in a static device array of 4 * FO_NOALLOC_MAX_N bytes + 512 bytes (16 MiB) that every
 * device the library runs on holds until the process ends.  The call allocates and frees nothing, on the host or
 * on the device, and enqueues kernels only.  Arguments, messages and amplitudes are those of fo_encode with a plan
 * made from the same parameters (bit for bit); diagnostic counters and per-kernel timing are not available.
 *   FO_ESIZE   the padded length exceeds FO_NOALLOC_MAX_N (fo_last_hip_error gives the figures)
 * All calls on one device share that device's array, which keeps the last call's contents (every call overwrites
 * what it reads, so nothing needs clearing): calls that overlap on one device, on whatever streams, race. */
int fo_encode_noalloc(const fo_params *params, const float *g, uint64_t round, uint32_t party, uint32_t flags,
                      uint64_t *bits, float *scales, void *hip_stream);

/* One whole iteration (Sec. 4, "At iteration t"): M encodes, server, one downlink decode and
 * x <- x - delta * g^d (eq. "workers update").  Gives the same bits and the same x as the three
 * calls above made by hand followed by the update.
 *   g   HOST array of M device pointers, each fp32[d];  x device fp32[d], updated in place
 * The intermediate messages stay in plan scratch; fo_step_messages exposes them.               */
int fo_step(fo_plan *plan, const float *const *g, float *x, float delta, uint64_t round,
            void *hip_stream);

/* fo_step with the iteration counter read on the device when the kernels run: round_dev is a device uint64 (8-byte
 * aligned).  For callers that capture the step into a HIP graph (problem sizes where the step is a chain of short
 * launches): the graph is captured once and replayed, the caller advancing *round_dev between replays (for example
 * with an increment kernel captured into the same graph).  eps and dither depend on the round, so replaying a
 * step captured with a fixed round would reuse them; this entry point exists to avoid that.  The library records
 * no memset and nothing but kernel launches on the stream. */
int fo_step_dev_round(fo_plan *plan, const float *const *g, float *x, float delta, const uint64_t *round_dev,
                      void *hip_stream);

/* Device pointers into plan scratch holding the messages of the last fo_step on this plan:
 * bits_up [M][W], scales_up [M][nblocks], bits_down [P][W], scales_down [nblocks].  Any out
 * argument may be NULL.  Valid until the next hot call on the plan. */
int fo_step_messages(fo_plan *plan, const uint64_t **bits_up, const float **scales_up,
                     const uint64_t **bits_down, const float **scales_down);

/* Optional counters (diagnostics; not part of the paper's method, but they watch its hypotheses).  While a stats
 * block is attached, every encode adds to it; the caller clears it (e.g. hipMemsetAsync) when it wants a fresh
 * count.  Attached counters cost the encodes a second sweep over their registers; detached (NULL, the default)
 * they cost nothing.
 *   clipped  coordinates with |(H_eps g)_i| > lambda: the complement of the event on which the flattening
 *            lemma (Lemma 3.6) holds and the quantiser is unbiased; 0 is the expected value for alpha >= 2
 *   near_tie coordinates with |(H_eps g)_i + tau_i| < 1e-6 lambda (first dither): where fp32 and fp64 may
 *            legitimately disagree on the sign
 * Index: worker n -> [n]; the server's re-encode -> [FO_MAX_WORKERS] (the zero-transform server of
 * FO_EPS_SHARED_ALL adds nothing: its vector is bounded by lambda <= lambda^s by construction). */
typedef struct {
    unsigned long long clipped[FO_MAX_WORKERS + 1];
    unsigned long long near_tie[FO_MAX_WORKERS + 1];
} fo_stats;
/* stats: device pointer (8-byte aligned) or NULL to detach. */
int fo_set_stats(fo_plan *plan, fo_stats *stats);

/* Optional per-kernel timing, for benchmarks (not part of the paper's method).  After
 * fo_profile_begin every kernel the hot calls enqueue on this plan is bracketed by two HIP events
 * on the caller's stream (the first call creates the events: it allocates, the hot calls still do
 * not).  fo_profile_end waits for the recorded work, writes one entry per kernel that ran into
 * the host array out[cap], sets *count and stops recording.  At most 8192 launches are recorded. */
typedef struct {
    char name[48];     /* kernel name as it appears in a rocprofv3 kernel trace (template form) */
    uint32_t launches;
    float total_ms;    /* sum of the launches' durations                                         */
} fo_kernel_time;
int fo_profile_begin(fo_plan *plan);
/* The same, bracketing only the launches of the named kernel (a name fo_profile_end reports): two event records
 * per launch of one kernel instead of all, for timing that kernel inside a region whose total time also counts
 * (events between kernels keep one from starting while the previous one drains: about 3 % on a 2 ms step). */
int fo_profile_begin_kernel(fo_plan *plan, const char *kernel_name);
int fo_profile_end(fo_plan *plan, fo_kernel_time *out, size_t cap, size_t *count);

#ifdef __cplusplus
}
#endif
#endif /* FO_H */
