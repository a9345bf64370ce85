/*
 * FO-SGD gradient codec -- plain CPU oracle (fp64).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * codec computes.  It shares no code, header, table or constant generator with the HIP library
 * and must never be called from the product path; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg load it.
 *
 * Paper: "Flattened one-bit stochastic gradient descent" (arXiv 2405.11095).  Every function
 * names the passage it follows.  All arithmetic is IEEE double; fp32 inputs are widened exactly.
 *
 * Readings of points on which the paper is silent (each also listed in the design notes):
 *   - d not a power of two: zero-pad to n = max(64, 2^ceil(log2 d)); the server works in R^n and
 *     only the final worker decode truncates to d.
 *   - blocked transform (not in the paper): block-diagonal direct sum of Hadamard bases of size
 *     b = 2^block_log2, one dither amplitude per block, eps and dither indexed by the global
 *     coordinate.  Sec. 3 Lemma "general flattening" (entries bounded by gamma = 1/sqrt(b))
 *     covers each block.
 *   - log is the natural logarithm (the flattening proof writes d = exp(log d)).
 *   - sign(0) = +1 (the quantizer-moment proof counts P(x + tau >= 0) for +1).
 *   - random numbers: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) keyed as described at
 *     orc_rng; the dither is the discrete symmetric grid u = (2r + 1 - 2^24) / 2^24, r = top 24
 *     bits of a 32-bit draw, so tau = lambda * u never equals 0 or +-lambda.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_DOMAIN_EPS 1u
#define ORC_DOMAIN_DITHER 2u
#define ORC_PARTY_SERVER 0xFFFFFFFFu
#define ORC_PARTY_ALL_WORKERS 0xFFFFFFFEu

#define ORC_DITHER_UNIFORM 0u
#define ORC_DITHER_NONE 1u
#define ORC_SCALE_BOUND 0u
#define ORC_SCALE_L2 1u
#define ORC_EPS_INDEPENDENT 0u
#define ORC_EPS_SHARED_WORKERS 1u
#define ORC_EPS_SHARED_ALL 2u
#define ORC_SERVER_SCALE_THM 0u
#define ORC_SERVER_SCALE_L2 1u
#define ORC_SERVER_SCALE_SUP 2u /* all-shared eps only: lambda^s = the workers' common amplitude */

typedef struct {
    uint64_t d;          /* logical gradient length                                  */
    uint32_t M;          /* number of workers (the paper's N)                        */
    uint32_t block_log2; /* 0: one transform over the padded vector; else b = 2^k    */
    uint32_t K;          /* averaging count of the server's quantizer (Def. 3.2)     */
    uint32_t dither;     /* ORC_DITHER_*                                             */
    uint32_t scale_rule; /* ORC_SCALE_*                                              */
    uint32_t eps_mode;   /* ORC_EPS_*                                                */
    double alpha, alpha_s, B;
    uint64_t seed;
    uint32_t server_scale; /* ORC_SERVER_SCALE_*                                        */
} orc_params;

/* ------------------------------------------------------------------------------------------ */
/* Random numbers                                                                             */
/* ------------------------------------------------------------------------------------------ */

/* Philox4x32 with 10 rounds, written from the construction in Salmon et al. (SC'11, Sec. 3.3):
 * each round multiplies words 0 and 2 by two fixed odd constants, keeps the low halves, and
 * xors the high halves with the other two words and the round key; the key is advanced by two
 * Weyl constants between rounds. */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The codec's stateless generator R(seed, domain, round, party, k, counter) -> 128 bits.
 * counter words: (counter, domain | k << 8, round mod 2^32, party); key: (seed mod 2^32,
 * (seed >> 32) xor (round >> 32)).  "uniformly distributed" and "independent" in Def. 3.2 and
 * Def. 3.5 are realised by distinct (domain, round, party, k, counter) tuples. */
void orc_rng(uint64_t seed, uint32_t domain, uint64_t round, uint32_t party, uint32_t k,
             uint32_t counter, uint32_t out[4])
{
    uint32_t ctr[4] = { counter, domain | (k << 8), (uint32_t)round, party };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) ^ (uint32_t)(round >> 32) };
    orc_philox4x32_10(ctr, key, out);
}

/* eps_i in {-1,+1} (Def. 3.5): one generator call covers 128 coordinates; coordinate i uses bit
 * (i mod 32) of word ((i / 32) mod 4) of call (i / 128); a set bit means eps_i = -1. */
int orc_eps(uint64_t seed, uint64_t round, uint32_t eps_party, uint64_t i)
{
    /* the last generator block is remembered per thread: consecutive coordinates share it */
    static _Thread_local struct { int valid; uint64_t seed, round; uint32_t party, counter, w[4]; } memo;
    uint32_t counter = (uint32_t)(i >> 7);
    if (!memo.valid || memo.seed != seed || memo.round != round || memo.party != eps_party ||
        memo.counter != counter) {
        orc_rng(seed, ORC_DOMAIN_EPS, round, eps_party, 0, counter, memo.w);
        memo.valid = 1; memo.seed = seed; memo.round = round; memo.party = eps_party;
        memo.counter = counter;
    }
    return ((memo.w[(i >> 5) & 3] >> (i & 31)) & 1u) ? -1 : +1;
}

/* eps_i for i = i0 .. i0 + n - 1 as +-1.0 (the same draws as orc_eps, one by one) */
void orc_eps_fill(uint64_t seed, uint64_t round, uint32_t eps_party, uint64_t i0, uint64_t n, double *out)
{
    for (uint64_t k = 0; k < n; ++k) out[k] = (double)orc_eps(seed, round, eps_party, i0 + k);
}

/* u_i in (-1,1) so that tau_i = lambda * u_i (Def. 3.2): one generator call covers the four
 * coordinates i = 256*q + 64*s + l (s = 0..3) with counter = 64*q + l; coordinate i takes word s.
 * The top 24 bits r give u = (2r + 1 - 2^24) / 2^24. */
double orc_dither_u(uint64_t seed, uint64_t round, uint32_t party, uint32_t k, uint64_t i)
{
    uint32_t w[4];
    uint32_t counter = (uint32_t)(((i >> 8) << 6) | (i & 63));
    orc_rng(seed, ORC_DOMAIN_DITHER, round, party, k, counter, w);
    uint32_t r = w[(i >> 6) & 3] >> 8;
    return (2.0 * (double)r + 1.0 - 16777216.0) / 16777216.0;
}

/* Which party's eps string a party uses (Sec. 4 draws one per worker and one for the server;
 * the shared modes are this build's variants). */
static uint32_t eps_party_of(uint32_t eps_mode, uint32_t party)
{
    if (eps_mode == ORC_EPS_INDEPENDENT) return party;
    if (eps_mode == ORC_EPS_SHARED_ALL) return ORC_PARTY_ALL_WORKERS;
    return party == ORC_PARTY_SERVER ? ORC_PARTY_SERVER : ORC_PARTY_ALL_WORKERS;
}
uint32_t orc_eps_party(uint32_t eps_mode, uint32_t party) { return eps_party_of(eps_mode, party); }

/* ------------------------------------------------------------------------------------------ */
/* Walsh-Hadamard transform (Def. 3.4)                                                        */
/* ------------------------------------------------------------------------------------------ */

/* Dense unnormalised matrix from the recursion H_0 = 1, H_k = [[H, H], [H, -H]]; row-major. */
void orc_sylvester(uint32_t k, double *H)
{
    uint64_t n = (uint64_t)1 << k;
    H[0] = 1.0;
    for (uint64_t m = 1; m < n; m <<= 1) {
        /* the top-left m x m block (stored with row stride n) is H_{log2 m}; fill the other three */
        for (uint64_t r = 0; r < m; ++r)
            for (uint64_t c = 0; c < m; ++c) {
                double v = H[r * n + c];
                H[r * n + (c + m)] = v;
                H[(r + m) * n + c] = v;
                H[(r + m) * n + (c + m)] = -v;
            }
    }
}

/* y = H x by the entry formula H_ij = (-1)^{popcount(i & j)} (the recursion unrolled). O(n^2). */
void orc_wht_dense(const double *x, double *y, uint64_t n)
{
    for (uint64_t i = 0; i < n; ++i) {
        double s = 0.0;
        for (uint64_t j = 0; j < n; ++j)
            s += (__builtin_popcountll(i & j) & 1) ? -x[j] : x[j];
        y[i] = s;
    }
}

/* Single entries of y = H x by the same entry formula: y[k] = sum_j (-1)^{popcount(idx[k] & j)} x[j].
 * O(n) per entry; lets a test check a few coordinates of a transform too long to run whole. */
void orc_wht_rows(const double *x, uint64_t n, const uint64_t *idx, uint64_t cnt, double *y)
{
    for (uint64_t k = 0; k < cnt; ++k) {
        const uint64_t i = idx[k];
        double s = 0.0;
        for (uint64_t j = 0; j < n; ++j)
            s += (__builtin_popcountll(i & j) & 1) ? -x[j] : x[j];
        y[k] = s;
    }
}

/* In-place unnormalised transform by butterflies, O(n log n) (Sec. 4, cost remark). */
void orc_fwht(double *x, uint64_t n)
{
    for (uint64_t h = 1; h < n; h <<= 1)
        for (uint64_t i = 0; i < n; i += 2 * h)
            for (uint64_t j = i; j < i + h; ++j) {
                double a = x[j], b = x[j + h];
                x[j] = a + b;
                x[j + h] = a - b;
            }
}

/* ------------------------------------------------------------------------------------------ */
/* Geometry                                                                                   */
/* ------------------------------------------------------------------------------------------ */

/* Transform length b, number of blocks and padded length ntot = b * nblocks. */
void orc_geometry(const orc_params *p, uint64_t *b, uint64_t *nblocks, uint64_t *ntot)
{
    uint64_t bb;
    if (p->block_log2 == 0) {
        bb = 64;
        while (bb < p->d) bb <<= 1;
        *nblocks = 1;
    } else {
        bb = (uint64_t)1 << p->block_log2;
        *nblocks = (p->d + bb - 1) / bb;
    }
    *b = bb;
    *ntot = bb * *nblocks;
}

/* ------------------------------------------------------------------------------------------ */
/* Quantizer (Def. 3.2)                                                                       */
/* ------------------------------------------------------------------------------------------ */

/* q_i = sum_{k<K} sign(z_i + tau_{k,i}) in {-K, -K+2, ..., K}, i.e. (K/lambda) Q_{lambda,K}(z)_i,
 * for the n coordinates with global indices i0 .. i0+n-1.  margin (optional) receives the
 * pre-quantisation value z_i + tau_{k,i} closest to zero over the K dithers (the one a rounding
 * difference would flip first); for K = 1 that is z_i + tau_{0,i}. */
void orc_quantize(const double *z, uint64_t n, uint64_t i0, double lam, uint32_t K,
                  uint32_t dither, uint64_t seed, uint64_t round, uint32_t party, int32_t *q,
                  double *margin)
{
    for (uint64_t l = 0; l < n; ++l) {
        int32_t s = 0;
        for (uint32_t k = 0; k < K; ++k) {
            double tau = 0.0;
            if (dither == ORC_DITHER_UNIFORM) tau = lam * orc_dither_u(seed, round, party, k, i0 + l);
            double t = z[l] + tau;
            if (margin && (k == 0 || fabs(t) < fabs(margin[l]))) margin[l] = t;
            s += (t >= 0.0) ? 1 : -1;
        }
        q[l] = s;
    }
}

/* word w, bit j <-> coordinate 64 w + j; a set bit <-> +1 ("stored using d bits", Sec. 4). */
void orc_pack(const int32_t *q, uint64_t n, uint64_t *bits)
{
    for (uint64_t w = 0; w < n / 64; ++w) {
        uint64_t v = 0;
        for (int j = 0; j < 64; ++j)
            if (q[64 * w + j] > 0) v |= (uint64_t)1 << j;
        bits[w] = v;
    }
}
void orc_unpack(const uint64_t *bits, uint64_t n, int32_t *q)
{
    for (uint64_t i = 0; i < n; ++i) q[i] = ((bits[i >> 6] >> (i & 63)) & 1u) ? 1 : -1;
}

/* ------------------------------------------------------------------------------------------ */
/* Encoder (Def. 3.7) and decoder (Def. 3.8)                                                  */
/* ------------------------------------------------------------------------------------------ */

/* Dither amplitude of Thm 5.5 for one block: lambda = alpha * B * sqrt(log n / n). */
double orc_lambda(double alpha, double B, uint64_t n)
{
    return alpha * B * sqrt(log((double)n) / (double)n);
}

/* E_{eps,lambda,K}(x) = (K/lambda) Q_{lambda,K}(H_eps x), per block, for blocks j0 .. j0+nj-1.
 * Blocks are independent, so a range of them can be encoded alone; every array below covers
 * that range only and is indexed from its first coordinate (block j0, coordinate j0*b).
 *   xs     input slice (already double): coordinates j0*b .. min(d, (j0+nj)*b) - 1
 *   lam    [nj]      force != 0: amplitudes to use; else written with the rule's value, where B
 *                    is p->B (BOUND) or the block's own l2 norm (L2)
 *   q      [nj*b]    integer code; bits [nj*b/64] packed signs when K == 1 (may be NULL)
 *   margin [nj*b]    optional z_i + tau_i;  z_out [nj*b] optional flattened vector H_eps x */
void orc_encode_blocks(const orc_params *p, const double *xs, uint64_t round, uint32_t party,
                       uint32_t K, int force, uint64_t j0, uint64_t nj, double *lam, int32_t *q,
                       uint64_t *bits, double *margin, double *z_out)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    uint32_t ep = eps_party_of(p->eps_mode, party);
    double *y = (double *)malloc(b * sizeof(double));
    double rs = 1.0 / sqrt((double)b);
    for (uint64_t jj = 0; jj < nj; ++jj) {
        uint64_t first = (j0 + jj) * b;                          /* global index of the block */
        double ss = 0.0;
        for (uint64_t l = 0; l < b; ++l) {
            uint64_t i = first + l;
            double v = (i < p->d) ? xs[jj * b + l] : 0.0;        /* zero padding beyond d */
            ss += v * v;
            y[l] = v * (double)orc_eps(p->seed, round, ep, i);   /* D_eps x */
        }
        orc_fwht(y, b);
        for (uint64_t l = 0; l < b; ++l) y[l] *= rs;             /* H = calH / sqrt(b) */
        if (!force) {
            double B = (p->scale_rule == ORC_SCALE_BOUND) ? p->B : sqrt(ss);
            lam[jj] = orc_lambda(p->alpha, B, b);
        }
        orc_quantize(y, b, first, lam[jj], K, p->dither, p->seed, round, party, q + jj * b,
                     margin ? margin + jj * b : NULL);
        if (z_out) memcpy(z_out + jj * b, y, b * sizeof(double));
    }
    if (bits && K == 1) orc_pack(q, nj * b, bits);
    free(y);
}

void orc_encode(const orc_params *p, const double *x, uint64_t round, uint32_t party, uint32_t K,
                int force, double *lam, int32_t *q, uint64_t *bits, double *margin, double *z_out)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    orc_encode_blocks(p, x, round, party, K, force, 0, nb, lam, q, bits, margin, z_out);
}

/* D_{eps,lambda,K}(q) = (lambda/K) D_eps H^T q, per block, for blocks j0 .. j0+nj-1; q [nj*b],
 * lam [nj] and out [nj*b] cover that range only (no truncation to d). */
void orc_decode_blocks(const orc_params *p, const int32_t *q, const double *lam, uint32_t K,
                       uint64_t round, uint32_t party, uint64_t j0, uint64_t nj, double *out)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    uint32_t ep = eps_party_of(p->eps_mode, party);
    double rs = 1.0 / sqrt((double)b);
    for (uint64_t jj = 0; jj < nj; ++jj) {
        double *y = out + jj * b;
        for (uint64_t l = 0; l < b; ++l) y[l] = (double)q[jj * b + l];
        orc_fwht(y, b);                                          /* H^T = H (symmetric) */
        for (uint64_t l = 0; l < b; ++l) {
            uint64_t i = (j0 + jj) * b + l;
            y[l] = (lam[jj] / (double)K) * (double)orc_eps(p->seed, round, ep, i) * (y[l] * rs);
        }
    }
}

void orc_decode(const orc_params *p, const int32_t *q, const double *lam, uint32_t K,
                uint64_t round, uint32_t party, double *out)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    orc_decode_blocks(p, q, lam, K, round, party, 0, nb, out);
}

/* ------------------------------------------------------------------------------------------ */
/* Server (Sec. 4: decode every worker, average, re-encode) and one full round                */
/* ------------------------------------------------------------------------------------------ */

/* Server amplitude of Thm 5.5, per block: lambda^s = alpha_s * lambda * sqrt(log n) with
 * lambda the largest worker amplitude of that block (or lambda itself, rule SUP, see below). */
void orc_server_lambda(const orc_params *p, const double *lam_up, double *lam_s)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    for (uint64_t j = 0; j < nb; ++j) {
        double m = 0.0;
        for (uint32_t n = 0; n < p->M; ++n)
            if (lam_up[(uint64_t)n * nb + j] > m) m = lam_up[(uint64_t)n * nb + j];
        /* a NaN amplitude must poison the result the way it poisons a sum */
        for (uint32_t n = 0; n < p->M; ++n)
            if (lam_up[(uint64_t)n * nb + j] != lam_up[(uint64_t)n * nb + j]) m = NAN;
        /* All-shared eps: the vector the server quantises is (lambda / M)(2 c - M), at most lambda in every
         * coordinate whatever eps is, and the quantiser of Def. 3.2 is unbiased as soon as ||z||_inf <= lambda^s
         * (first moment of the quantiser, Appendix): the amplitude lambda itself is then admissible. */
        if (p->server_scale == ORC_SERVER_SCALE_SUP) lam_s[j] = m;
        else lam_s[j] = p->alpha_s * m * sqrt(log((double)b));
    }
}

/* gbar = (1/M) sum_n D_{eps_n,lambda_n}(q_n)  (eq. server average), then the (eps^s, lambda^s, K)
 * encoder applied to gbar.  bits_up [M][ntot/64], lam_up [M][nb]. */
void orc_server(const orc_params *p, const uint64_t *bits_up, const double *lam_up, uint64_t round,
                double *gbar, int force_s, double *lam_s, int32_t *q_down, uint64_t *bits_down,
                double *margin)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    int32_t *q = (int32_t *)malloc(ntot * sizeof(int32_t));
    double *dec = (double *)malloc(ntot * sizeof(double));
    for (uint64_t i = 0; i < ntot; ++i) gbar[i] = 0.0;
    for (uint32_t n = 0; n < p->M; ++n) {
        orc_unpack(bits_up + (uint64_t)n * (ntot / 64), ntot, q);
        orc_decode(p, q, lam_up + (uint64_t)n * nb, 1, round, n, dec);
        for (uint64_t i = 0; i < ntot; ++i) gbar[i] += dec[i];
    }
    for (uint64_t i = 0; i < ntot; ++i) gbar[i] /= (double)p->M;
    free(q);
    free(dec);
    if (!force_s) {
        if (p->server_scale == ORC_SERVER_SCALE_L2) {
            /* The smallest amplitude the server lemma in the proof of Thm 5.5 admits: it only uses
             * lambda^s >= alpha_s sqrt(log n / n) ||w|| for the vector w being encoded, here gbar (per block). */
            for (uint64_t j = 0; j < nb; ++j) {
                double s2 = 0.0;
                for (uint64_t l = 0; l < b; ++l) s2 += gbar[j * b + l] * gbar[j * b + l];
                lam_s[j] = orc_lambda(p->alpha_s, sqrt(s2), b);
            }
        } else {
            orc_server_lambda(p, lam_up, lam_s);
        }
    }
    /* the server encodes a vector of length ntot: same geometry, logical length ntot */
    orc_params ps = *p;
    ps.d = ntot;
    orc_encode(&ps, gbar, round, ORC_PARTY_SERVER, p->K, 1, lam_s, q_down, bits_down, margin, NULL);
}

typedef struct {
    const orc_params *p;
    const float *g;
    uint64_t round;
    uint32_t party;
    double *lam;
    uint64_t *bits;
} enc_job;

static void *enc_thread(void *arg)
{
    enc_job *jb = (enc_job *)arg;
    uint64_t b, nb, ntot;
    orc_geometry(jb->p, &b, &nb, &ntot);
    double *x = (double *)malloc(jb->p->d * sizeof(double));
    int32_t *q = (int32_t *)malloc(ntot * sizeof(int32_t));
    for (uint64_t i = 0; i < jb->p->d; ++i) x[i] = (double)jb->g[i];
    orc_encode(jb->p, x, jb->round, jb->party, 1, 0, jb->lam, q, jb->bits, NULL, NULL);
    free(x);
    free(q);
    return NULL;
}

/* One FO-SGD iteration (Sec. 4, "At iteration t"): M worker encodes (run on up to nthreads
 * threads, one worker per thread), server decode + average + re-encode, worker decode of the
 * downlink, x <- x - delta * g^d.  g: M pointers to fp32[d]; x: double[d] in place.
 * Optional outputs (may be NULL): bits_up [M][W], lam_up [M][nb], gbar [ntot], bits_down [W],
 * lam_s [nb], gd [d]. */
void orc_round(const orc_params *p, const float *const *g, double *x, double delta, uint64_t round,
               int nthreads, uint64_t *bits_up_o, double *lam_up_o, double *gbar_o,
               uint64_t *bits_down_o, double *lam_s_o, double *gd_o)
{
    uint64_t b, nb, ntot;
    orc_geometry(p, &b, &nb, &ntot);
    uint64_t W = ntot / 64;
    uint64_t *bits_up = bits_up_o ? bits_up_o : (uint64_t *)malloc(p->M * W * sizeof(uint64_t));
    double *lam_up = lam_up_o ? lam_up_o : (double *)malloc(p->M * nb * sizeof(double));
    double *gbar = gbar_o ? gbar_o : (double *)malloc(ntot * sizeof(double));
    uint64_t *bits_down = bits_down_o ? bits_down_o : (uint64_t *)malloc(W * sizeof(uint64_t));
    double *lam_s = lam_s_o ? lam_s_o : (double *)malloc(nb * sizeof(double));

    enc_job *jobs = (enc_job *)malloc(p->M * sizeof(enc_job));
    pthread_t *th = (pthread_t *)malloc(p->M * sizeof(pthread_t));
    if (nthreads < 1) nthreads = 1;
    for (uint32_t n0 = 0; n0 < p->M; n0 += (uint32_t)nthreads) {
        uint32_t n1 = n0 + (uint32_t)nthreads < p->M ? n0 + (uint32_t)nthreads : p->M;
        for (uint32_t n = n0; n < n1; ++n) {
            jobs[n] = (enc_job){ p, g[n], round, n, lam_up + (uint64_t)n * nb, bits_up + (uint64_t)n * W };
            pthread_create(&th[n], NULL, enc_thread, &jobs[n]);
        }
        for (uint32_t n = n0; n < n1; ++n) pthread_join(th[n], NULL);
    }
    free(jobs);
    free(th);

    int32_t *qd = (int32_t *)malloc(ntot * sizeof(int32_t));
    orc_server(p, bits_up, lam_up, round, gbar, 0, lam_s, qd, p->K == 1 ? bits_down : NULL, NULL);
    double *gd = (double *)malloc(ntot * sizeof(double));
    orc_decode(p, qd, lam_s, p->K, round, ORC_PARTY_SERVER, gd);
    for (uint64_t i = 0; i < p->d; ++i) x[i] -= delta * gd[i];
    if (gd_o) memcpy(gd_o, gd, p->d * sizeof(double));
    free(gd);
    free(qd);
    if (!bits_up_o) free(bits_up);
    if (!lam_up_o) free(lam_up);
    if (!gbar_o) free(gbar);
    if (!bits_down_o) free(bits_down);
    if (!lam_s_o) free(lam_s);
}
