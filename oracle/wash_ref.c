/*
 * CPU oracle for the WASH population-update path (arXiv 2405.17517).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT PRODUCT CODE.  It is the slow, plain
 * definition of what the GPU library must compute.  Only the tests, the smoke
 * check and the CPU-baseline leg of the benchmark may load it.  It shares no
 * source, header, table or helper with the HIP library.
 *
 * What is written out here, and the passage of the paper each part follows:
 *   - shuffle step            : Sec. 3, Eq. 3 and Alg. 1 (shuffling step);
 *                               permutation uniform on all of S_N and
 *                               independent of the Bernoulli draw (text
 *                               below Eq. 3); optimizer state moved with its
 *                               weight (WASH+Opt, Sec. 4 "Training methods")
 *   - layer-wise probability  : Sec. 3, Eq. 6 (and the constant / increasing
 *                               schedules of the appendix ablation table)
 *   - uniform average         : Alg. 1 output line; consensus definition
 *                               below Eq. 1
 *   - PAPA EMA                : Sec. 3, Eq. 1
 *   - distance to consensus   : the quantity of Eq. 2, Eq. 5 and Fig. 2
 *   - weighted average        : convex combinations of the models (appendix,
 *                               interpolation heatmaps)
 *
 * The paper fixes only the LAW of the shuffle.  A bit-exact comparison needs
 * one concrete random stream; the one defined here ("stream v1") is this
 * repository's own choice and the distributional pins in the tests are what
 * tie it back to the paper:
 *
 *   PRF        Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11).
 *   key        (low 32 bits of seed, high 32 bits of seed)
 *   mask word  for coordinate g (position in the flat row, 0 <= g < P):
 *                word (g mod 4) of Philox(key, (lo32(g/4), hi32(g/4), lo32(step), 0))
 *              coordinate g is selected  <=>  word < T,  T = round(p * 2^32)
 *              as a 64-bit compare (p = 1 selects always, p = 0 never).
 *   perm words w_t, t = 0 .. N-2, for a selected g:
 *                word (t mod 4) of Philox(key, (lo32(g), hi32(g), lo32(step), 1 + t/4))
 *   Fisher-Yates, descending: perm = identity; for i = N-1 .. 1 with
 *              t = N-1-i:  j = (w_t * (i+1)) >> 32;  swap(perm[i], perm[j]).
 *   gather     new[n] = old[perm[n]]  (Eq. 3 as written: theta_hat_n = theta_{pi(n)}).
 *
 * Parity status: the invariants, closed forms and known answers this file is
 * pinned to are in tests/test_oracle_*.py.  The one thing that cannot be
 * pinned to the paper is the exact bit stream of the shuffle (the paper gives
 * none): "parity unpinned" for the identity of the stream, pinned for its law.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define WASH_REF_MAX_N 32u

typedef struct {
    uint64_t offset; /* first coordinate of the segment inside a row */
    uint64_t length; /* number of coordinates */
    double p;        /* shuffle probability of every coordinate in it */
} wash_ref_segment;

/* ------------------------------------------------------------------------ */
/* Philox4x32-10, from the published round function and key schedule.        */

void wash_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(prod0 >> 32), lo0 = (uint32_t)prod0;
        uint32_t hi1 = (uint32_t)(prod1 >> 32), lo1 = (uint32_t)prod1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; /* key bump after every round; the 10th bump is unused */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------ */
/* Pieces of the random stream, exported so that tests can pin each alone.   */

/* T = round(p * 2^32) in IEEE double, as an integer in [0, 2^32]. */
uint64_t wash_ref_threshold(double p)
{
    double t = floor(p * 4294967296.0 + 0.5);
    if (t < 0.0) t = 0.0;
    if (t > 4294967296.0) t = 4294967296.0;
    return (uint64_t)t;
}

/* The 32-bit mask word of coordinate g at (seed, step). */
uint32_t wash_ref_mask_word(uint64_t seed, uint64_t step, uint64_t g)
{
    uint64_t quad = g >> 2;
    uint32_t ctr[4] = { (uint32_t)quad, (uint32_t)(quad >> 32), (uint32_t)step, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    wash_ref_philox4x32_10(ctr, key, out);
    return out[g & 3u];
}

/* The N-1 permutation words of coordinate g at (seed, step). */
void wash_ref_perm_words(uint64_t seed, uint64_t step, uint64_t g, uint32_t N, uint32_t *w)
{
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    for (uint32_t t = 0; t + 1 < N; ++t) {
        uint32_t ctr[4] = { (uint32_t)g, (uint32_t)(g >> 32), (uint32_t)step, 1u + (t >> 2) };
        uint32_t out[4];
        wash_ref_philox4x32_10(ctr, key, out);
        w[t] = out[t & 3u];
    }
}

/* Descending Fisher-Yates driven by N-1 given words. */
void wash_ref_fisher_yates(const uint32_t *w, uint32_t N, uint32_t *perm)
{
    for (uint32_t n = 0; n < N; ++n) perm[n] = n;
    for (uint32_t t = 0; t + 1 < N; ++t) {
        uint32_t i = N - 1u - t;
        uint32_t j = (uint32_t)(((uint64_t)w[t] * (uint64_t)(i + 1u)) >> 32);
        uint32_t tmp = perm[i];
        perm[i] = perm[j];
        perm[j] = tmp;
    }
}

/* pi_g at (seed, step): what the shuffle applies to coordinate g if selected. */
int wash_ref_permutation(uint64_t seed, uint64_t step, uint64_t g, uint32_t N, uint32_t *perm)
{
    uint32_t w[WASH_REF_MAX_N];
    if (N == 0 || N > WASH_REF_MAX_N) return -1;
    wash_ref_perm_words(seed, step, g, N, w);
    wash_ref_fisher_yates(w, N, perm);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Eq. 6 and its two ablation variants.                                       */

int wash_layer_probs_ref(double p, uint32_t L, int schedule, double *out)
{
    if (!(p >= 0.0 && p <= 1.0) || L == 0 || out == NULL) return -1;
    if (schedule < 0 || schedule > 2) return -1;
    for (uint32_t l = 0; l < L; ++l) {
        double frac = (L == 1) ? 0.0 : (double)l / (double)(L - 1u);
        if (schedule == 0) out[l] = p * (1.0 - frac);      /* Eq. 6: p at layer 0, 0 at layer L-1 */
        else if (schedule == 1) out[l] = p;                /* constant */
        else out[l] = (L == 1) ? p : p * frac;             /* increasing: 0 at layer 0, p at L-1 */
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* The shuffle step.                                                          */

static int check_segments(uint64_t P, const wash_ref_segment *segs, uint32_t nsegs)
{
    uint64_t prev_end = 0;
    for (uint32_t s = 0; s < nsegs; ++s) {
        if (!(segs[s].p >= 0.0 && segs[s].p <= 1.0)) return -1;
        if (segs[s].offset < prev_end) return -1;
        if (segs[s].offset > P || segs[s].length > P - segs[s].offset) return -1;
        prev_end = segs[s].offset + segs[s].length;
    }
    return 0;
}

/*
 * Shuffle the coordinates g in [g_begin, g_end) of a population whose columns
 * g_begin.. are stored in a window: value of model n at coordinate g sits at
 * params[n * row_stride + (g - g_begin)].  g is always the GLOBAL coordinate
 * (the random stream is addressed by it).  With g_begin = 0, g_end = P and
 * row_stride = P the window is the whole [N, P] population.
 */
int wash_shuffle_ref_window(float *params, float *momentum, uint32_t N, uint64_t P,
                            uint64_t row_stride, uint64_t g_begin, uint64_t g_end,
                            const wash_ref_segment *segs, uint32_t nsegs,
                            uint64_t seed, uint64_t step, uint64_t *selected_count)
{
    if (params == NULL || N == 0 || N > WASH_REF_MAX_N || P == 0) return -1;
    if (g_begin > g_end || g_end > P || step >= 4294967296ull) return -1;
    if (nsegs > 0 && segs == NULL) return -1;
    if (check_segments(P, segs, nsegs) != 0) return -1;

    uint32_t *vals = (uint32_t *)params;   /* values are moved as raw bits */
    uint32_t *moms = (uint32_t *)momentum;
    uint64_t count = 0;

    for (uint32_t s = 0; s < nsegs; ++s) {
        uint64_t T = wash_ref_threshold(segs[s].p);
        uint64_t lo = segs[s].offset, hi = segs[s].offset + segs[s].length;
        if (lo < g_begin) lo = g_begin;
        if (hi > g_end) hi = g_end;
        for (uint64_t g = lo; g < hi; ++g) {
            /* Bernoulli(p_s), one draw per coordinate, shared by all N models */
            uint32_t u = wash_ref_mask_word(seed, step, g);
            if (!((uint64_t)u < T)) continue;
            ++count;
            /* pi_g, uniform on S_N, from words independent of the mask word */
            uint32_t perm[WASH_REF_MAX_N];
            wash_ref_permutation(seed, step, g, N, perm);
            /* theta_hat[n] = theta[pi(n)], same pi for the optimizer state */
            uint32_t old[WASH_REF_MAX_N];
            uint64_t col = g - g_begin;
            for (uint32_t n = 0; n < N; ++n) old[n] = vals[(uint64_t)n * row_stride + col];
            for (uint32_t n = 0; n < N; ++n) vals[(uint64_t)n * row_stride + col] = old[perm[n]];
            if (moms != NULL) {
                for (uint32_t n = 0; n < N; ++n) old[n] = moms[(uint64_t)n * row_stride + col];
                for (uint32_t n = 0; n < N; ++n) moms[(uint64_t)n * row_stride + col] = old[perm[n]];
            }
        }
    }
    if (selected_count != NULL) *selected_count += count;
    return 0;
}

int wash_shuffle_ref(float *params, float *momentum, uint32_t N, uint64_t P,
                     const wash_ref_segment *segs, uint32_t nsegs,
                     uint64_t seed, uint64_t step, uint64_t *selected_count)
{
    return wash_shuffle_ref_window(params, momentum, N, P, P, 0, P, segs, nsegs, seed, step,
                                   selected_count);
}

/* ------------------------------------------------------------------------ */
/*
 * The same shuffle step with a second mask stream, "gap" (stream v2).
 *
 * Law: identical to Eq. 3 -- every coordinate of a segment is selected
 * independently with the segment's probability p, then permuted by pi_g exactly
 * as above.  Only the way the Bernoulli mask is drawn differs: instead of one
 * draw per coordinate, the distances between successive selected coordinates
 * are drawn.  For iid Bernoulli(p) trials the number of trials up to and
 * including the next success is geometric, P(gap > k) = (1-p)^k, and by
 * inversion  gap = 1 + floor(log2(u) / log2(1-p))  for u uniform on (0, 1].
 * Because the geometric law has no memory, restarting the walk at fixed places
 * leaves the trials iid; the walk restarts at every multiple of 1024
 * coordinates and at every segment start, which makes the stream addressable
 * (a piece depends on nothing before it).  The work is proportional to the
 * number of selected coordinates instead of the number of coordinates.
 *
 * Definition (this repository's own; the paper fixes the law only):
 *   - zero-length segments are dropped and neighbours that touch and have the
 *     same p (same double) are merged; segments with p = 0 select nothing, and
 *     neither do segments whose p is so small that 1 - p rounds to 1 in double
 *     (p <= 2^-54: log2(1 - p) would be 0 and the inversion meaningless; the
 *     Bernoulli(p) law of Eq. 3 is then met to within 2^-54 per coordinate,
 *     far inside the 2^-33 of the other stream's threshold);
 *   - a merged segment [a, b) is cut into pieces [s, e) at the multiples of 1024;
 *   - in a piece, pos = s - 1; for d = 0, 1, 2, ...:
 *       U_d  = the top 53 bits of the 64-bit number (hi = word 2(d mod 2),
 *              lo = word 2(d mod 2)+1) of Philox(key, (lo32(s), hi32(s),
 *              lo32(step), 0x80000000 + d/2));
 *       gap  = 1 + floor((wash_ref_log2(U_d + 1) - 53) * inv), capped at 2048,
 *              inv = 1 / wash_ref_log2(1 - p)  (inv = 0 for p = 1);
 *       pos += gap; stop if pos >= e; coordinate pos is selected.
 *   - pi_g and the gather are those of stream v1.
 * wash_ref_log2 is a fixed sequence of IEEE double operations (below), so that
 * another implementation can reproduce it bit for bit.
 */
#define WASH_REF_PIECE 1024u

/* log2 of a positive finite normal double, as a fixed sequence of IEEE
   operations: split x = m * 2^e with m in (sqrt(1/2), sqrt(2)], then
   ln m = 2 atanh(s), s = (m-1)/(m+1), by its odd series up to s^21. */
double wash_ref_log2(double x)
{
    uint64_t bits;
    memcpy(&bits, &x, sizeof bits);
    int e = (int)((bits >> 52) & 0x7FFu) - 1023;
    bits = (bits & 0x000FFFFFFFFFFFFFull) | 0x3FF0000000000000ull;
    double m;
    memcpy(&m, &bits, sizeof m);
    if (m > 1.4142135623730951) { m = m * 0.5; e += 1; }
    double s = (m - 1.0) / (m + 1.0);
    double z = s * s;
    double poly = 1.0 / 21.0;
    poly = poly * z + 1.0 / 19.0;
    poly = poly * z + 1.0 / 17.0;
    poly = poly * z + 1.0 / 15.0;
    poly = poly * z + 1.0 / 13.0;
    poly = poly * z + 1.0 / 11.0;
    poly = poly * z + 1.0 / 9.0;
    poly = poly * z + 1.0 / 7.0;
    poly = poly * z + 1.0 / 5.0;
    poly = poly * z + 1.0 / 3.0;
    poly = poly * z + 1.0;
    double t = s * poly;
    double ln_m = t + t;
    return (double)e + ln_m * 1.4426950408889634;
}

/* 1 / log2(1 - p) for 0 < p < 1 (negative); 0 for p = 1. */
double wash_ref_gap_scale(double p)
{
    if (p >= 1.0) return 0.0;
    return 1.0 / wash_ref_log2(1.0 - p);
}

/* The d-th 53-bit uniform of the piece that starts at coordinate s. */
uint64_t wash_ref_gap_uniform(uint64_t seed, uint64_t step, uint64_t s, uint32_t d)
{
    uint32_t ctr[4] = { (uint32_t)s, (uint32_t)(s >> 32), (uint32_t)step, 0x80000000u + (d >> 1) };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    wash_ref_philox4x32_10(ctr, key, out);
    uint64_t w = ((uint64_t)out[2u * (d & 1u)] << 32) | (uint64_t)out[2u * (d & 1u) + 1u];
    return w >> 11;
}

/* Geometric gap (>= 1, capped at 2048) from a 53-bit uniform U and inv = 1/log2(1-p). */
uint32_t wash_ref_gap(uint64_t U, double inv)
{
    double L = wash_ref_log2((double)(U + 1u)) - 53.0; /* log2 of u = (U+1)/2^53, in [-53, 0] */
    double q = L * inv;                                /* >= 0 for the inv of a probability */
    if (!(q < 2047.0)) q = 2047.0;                     /* also NaN */
    if (q < 0.0) q = 0.0;
    return 1u + (uint32_t)floor(q);
}

/* Walks the gap stream over the pieces that start inside [g_begin, g_end) and calls
   visit(ctx, g) for every selected coordinate g, in ascending order. */
typedef void (*gap_visit_fn)(void *ctx, uint64_t g);

static void gap_walk(uint64_t g_begin, uint64_t g_end, const wash_ref_segment *segs, uint32_t nsegs,
                     uint64_t seed, uint64_t step, gap_visit_fn visit, void *ctx)
{
    uint32_t k = 0;
    while (k < nsegs) {
        /* next merged segment [a, b) with probability p */
        while (k < nsegs && segs[k].length == 0) ++k;
        if (k == nsegs) break;
        uint64_t a = segs[k].offset, b = segs[k].offset + segs[k].length;
        double p = segs[k].p;
        ++k;
        while (k < nsegs && (segs[k].length == 0 || (segs[k].offset == b && segs[k].p == p))) {
            if (segs[k].length != 0) b = segs[k].offset + segs[k].length;
            ++k;
        }
        if (p == 0.0 || 1.0 - p == 1.0) continue;
        double inv = wash_ref_gap_scale(p);

        for (uint64_t s = a; s < b; ) {
            uint64_t e = (s / WASH_REF_PIECE + 1u) * WASH_REF_PIECE; /* next multiple of 1024 */
            if (e > b) e = b;
            if (s >= g_begin && s < g_end) {
                uint64_t pos = s - 1u; /* wraps for s = 0; the first gap (>= 1) brings it back */
                for (uint32_t d = 0;; ++d) {
                    pos += wash_ref_gap(wash_ref_gap_uniform(seed, step, s, d), inv);
                    if (pos >= e) break;
                    visit(ctx, pos);
                }
            }
            s = e;
        }
    }
}

static int gap_window_ok(uint64_t P, uint64_t g_begin, uint64_t g_end)
{
    /* pieces are whole inside or outside a window only if it is cut on the piece grid */
    if (g_begin > g_end || g_end > P) return 0;
    if (g_begin % WASH_REF_PIECE != 0) return 0;
    if (g_end % WASH_REF_PIECE != 0 && g_end != P) return 0;
    return 1;
}

typedef struct {
    uint32_t *vals, *moms;
    uint32_t N;
    uint64_t row_stride, g_begin, seed, step, count;
} gap_shuffle_ctx;

static void gap_shuffle_visit(void *vctx, uint64_t g)
{
    gap_shuffle_ctx *c = (gap_shuffle_ctx *)vctx;
    uint32_t perm[WASH_REF_MAX_N], old[WASH_REF_MAX_N];
    ++c->count;
    wash_ref_permutation(c->seed, c->step, g, c->N, perm);   /* pi_g as in stream v1 */
    uint64_t col = g - c->g_begin;
    for (uint32_t n = 0; n < c->N; ++n) old[n] = c->vals[(uint64_t)n * c->row_stride + col];
    for (uint32_t n = 0; n < c->N; ++n) c->vals[(uint64_t)n * c->row_stride + col] = old[perm[n]];
    if (c->moms != NULL) {
        for (uint32_t n = 0; n < c->N; ++n) old[n] = c->moms[(uint64_t)n * c->row_stride + col];
        for (uint32_t n = 0; n < c->N; ++n) c->moms[(uint64_t)n * c->row_stride + col] = old[perm[n]];
    }
}

int wash_shuffle_gap_ref_window(float *params, float *momentum, uint32_t N, uint64_t P,
                                uint64_t row_stride, uint64_t g_begin, uint64_t g_end,
                                const wash_ref_segment *segs, uint32_t nsegs,
                                uint64_t seed, uint64_t step, uint64_t *selected_count)
{
    if (params == NULL || N == 0 || N > WASH_REF_MAX_N || P == 0) return -1;
    if (step >= 4294967296ull || !gap_window_ok(P, g_begin, g_end)) return -1;
    if (nsegs > 0 && segs == NULL) return -1;
    if (check_segments(P, segs, nsegs) != 0) return -1;
    gap_shuffle_ctx c = { (uint32_t *)params, (uint32_t *)momentum, N, row_stride, g_begin, seed, step, 0 };
    gap_walk(g_begin, g_end, segs, nsegs, seed, step, gap_shuffle_visit, &c);
    if (selected_count != NULL) *selected_count += c.count;
    return 0;
}

/* The Bernoulli mask of the gap stream alone: mask[g] = 1 for every selected g, else untouched. */
static void gap_mask_visit(void *vctx, uint64_t g) { ((uint8_t *)vctx)[g] = 1u; }

int wash_ref_gap_mask(uint8_t *mask, uint64_t P, const wash_ref_segment *segs, uint32_t nsegs,
                      uint64_t seed, uint64_t step)
{
    if (mask == NULL || P == 0 || step >= 4294967296ull) return -1;
    if (nsegs > 0 && segs == NULL) return -1;
    if (check_segments(P, segs, nsegs) != 0) return -1;
    gap_walk(0, P, segs, nsegs, seed, step, gap_mask_visit, mask);
    return 0;
}

int wash_shuffle_gap_ref(float *params, float *momentum, uint32_t N, uint64_t P,
                         const wash_ref_segment *segs, uint32_t nsegs,
                         uint64_t seed, uint64_t step, uint64_t *selected_count)
{
    return wash_shuffle_gap_ref_window(params, momentum, N, P, P, 0, P, segs, nsegs, seed, step,
                                       selected_count);
}

/* ------------------------------------------------------------------------ */
/* Uniform average and PAPA EMA: the definitions in fp64, rounded once.      */

int wash_average_ref(const float *params, float *out, uint32_t N, uint64_t P)
{
    if (params == NULL || out == NULL || N == 0 || P == 0) return -1;
    for (uint64_t g = 0; g < P; ++g) {
        double sum = 0.0;
        for (uint32_t n = 0; n < N; ++n) sum += (double)params[(uint64_t)n * P + g];
        out[g] = (float)(sum / (double)N);
    }
    return 0;
}

int papa_ema_ref(float *params, uint32_t N, uint64_t P, float alpha)
{
    if (params == NULL || N == 0 || P == 0 || !(alpha == alpha)) return -1;
    double a = (double)alpha;
    for (uint64_t g = 0; g < P; ++g) {
        double sum = 0.0;
        for (uint32_t n = 0; n < N; ++n) sum += (double)params[(uint64_t)n * P + g];
        double mean = sum / (double)N; /* consensus of the values BEFORE the update */
        for (uint32_t n = 0; n < N; ++n) {
            double x = (double)params[(uint64_t)n * P + g];
            params[(uint64_t)n * P + g] = (float)(a * x + (1.0 - a) * mean);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/*
 * Distance to the consensus (the paper's diagnostic: Fig. 2 plots
 * (1/N) sum_n ||theta_n - mean||, Eq. 2 and Eq. 5 are statements about
 * sum_n ||theta_n - mean||^2; the layer-schedule figure uses slices of the
 * parameter vector).  out[n] = sum over g in [g_begin, g_end) of
 * (theta[n][g] - mean[g])^2, everything in fp64, mean[g] = (sum_n theta[n][g]) / N
 * unrounded.  The caller takes square roots / averages over n as needed.
 */
int wash_consensus_sqdist_ref(const float *params, uint32_t N, uint64_t P,
                              uint64_t g_begin, uint64_t g_end, double *out)
{
    if (params == NULL || out == NULL || N == 0 || P == 0) return -1;
    if (g_begin > g_end || g_end > P) return -1;
    for (uint32_t n = 0; n < N; ++n) out[n] = 0.0;
    for (uint64_t g = g_begin; g < g_end; ++g) {
        double sum = 0.0;
        for (uint32_t n = 0; n < N; ++n) sum += (double)params[(uint64_t)n * P + g];
        double mean = sum / (double)N;
        for (uint32_t n = 0; n < N; ++n) {
            double d = (double)params[(uint64_t)n * P + g] - mean;
            out[n] += d * d;
        }
    }
    return 0;
}

/*
 * Weighted combination of the models (the interpolation study of the appendix
 * evaluates arbitrary convex combinations; GreedySoup-style soups average a
 * subset): out[g] = sum_n w[n] * theta[n][g], products and sum in fp64 in
 * ascending n, rounded once to fp32.  w = (1/N, ..., 1/N) is the uniform
 * average up to the rounding of 1/N.
 */
int wash_weighted_average_ref(const float *params, const double *w, float *out, uint32_t N, uint64_t P)
{
    if (params == NULL || w == NULL || out == NULL || N == 0 || P == 0) return -1;
    for (uint32_t n = 0; n < N; ++n) if (!(w[n] == w[n]) || w[n] - w[n] != 0.0) return -1; /* NaN or infinite */
    for (uint64_t g = 0; g < P; ++g) {
        double sum = 0.0;
        for (uint32_t n = 0; n < N; ++n) sum += w[n] * (double)params[(uint64_t)n * P + g];
        out[g] = (float)sum;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/*
 * The same shuffle, with the coordinate range cut into contiguous pieces, one
 * per thread.  Every piece runs wash_shuffle_ref_window above unchanged; the
 * stream is addressed by (seed, step, g) so the bits do not depend on the cut.
 * Used to time the oracle on all host cores and to keep full-size parity
 * tests short.
 */
typedef struct {
    float *params, *momentum;
    uint32_t N;
    uint64_t P, g_begin, g_end;
    const wash_ref_segment *segs;
    uint32_t nsegs;
    uint64_t seed, step, count;
    int status;
    int gap_stream;
} shuffle_job;

static void *shuffle_job_run(void *arg)
{
    shuffle_job *j = (shuffle_job *)arg;
    j->count = 0;
    /* the window here is the whole population (stride P, columns from 0), but
       only coordinates in [g_begin, g_end) are visited */
    if (j->g_begin == j->g_end) { j->status = 0; return NULL; }
    if (j->gap_stream)
        j->status = wash_shuffle_gap_ref_window(j->params + j->g_begin,
                                                j->momentum ? j->momentum + j->g_begin : NULL,
                                                j->N, j->P, j->P, j->g_begin, j->g_end,
                                                j->segs, j->nsegs, j->seed, j->step, &j->count);
    else
        j->status = wash_shuffle_ref_window(j->params + j->g_begin,
                                            j->momentum ? j->momentum + j->g_begin : NULL,
                                            j->N, j->P, j->P, j->g_begin, j->g_end,
                                            j->segs, j->nsegs, j->seed, j->step, &j->count);
    return NULL;
}

static int shuffle_mt(int gap_stream, float *params, float *momentum, uint32_t N, uint64_t P,
                      const wash_ref_segment *segs, uint32_t nsegs,
                      uint64_t seed, uint64_t step, uint64_t *selected_count,
                      uint32_t nthreads)
{
    if (nthreads == 0) return -1;
    if (nthreads > 256) nthreads = 256;
    if (params == NULL || N == 0 || N > WASH_REF_MAX_N || P == 0) return -1;
    shuffle_job jobs[256];
    pthread_t tids[256];
    for (uint32_t k = 0; k < nthreads; ++k) {
        shuffle_job *j = &jobs[k];
        j->params = params; j->momentum = momentum; j->N = N; j->P = P;
        /* cuts on multiples of 1024 (the piece grid of the gap stream; harmless for v1) */
        j->g_begin = (uint64_t)(((__uint128_t)P * k) / nthreads) / WASH_REF_PIECE * WASH_REF_PIECE;
        j->g_end = (uint64_t)(((__uint128_t)P * (k + 1u)) / nthreads) / WASH_REF_PIECE * WASH_REF_PIECE;
        if (k + 1u == nthreads) j->g_end = P;
        j->gap_stream = gap_stream;
        j->segs = segs; j->nsegs = nsegs; j->seed = seed; j->step = step;
        j->count = 0; j->status = 0;
    }
    for (uint32_t k = 0; k < nthreads; ++k)
        if (pthread_create(&tids[k], NULL, shuffle_job_run, &jobs[k]) != 0) {
            for (uint32_t m = 0; m < k; ++m) pthread_join(tids[m], NULL);
            return -2;
        }
    int status = 0;
    uint64_t count = 0;
    for (uint32_t k = 0; k < nthreads; ++k) {
        pthread_join(tids[k], NULL);
        if (jobs[k].status != 0) status = jobs[k].status;
        count += jobs[k].count;
    }
    if (status == 0 && selected_count != NULL) *selected_count += count;
    return status;
}

int wash_shuffle_ref_mt(float *params, float *momentum, uint32_t N, uint64_t P,
                        const wash_ref_segment *segs, uint32_t nsegs,
                        uint64_t seed, uint64_t step, uint64_t *selected_count,
                        uint32_t nthreads)
{
    return shuffle_mt(0, params, momentum, N, P, segs, nsegs, seed, step, selected_count, nthreads);
}

int wash_shuffle_gap_ref_mt(float *params, float *momentum, uint32_t N, uint64_t P,
                            const wash_ref_segment *segs, uint32_t nsegs,
                            uint64_t seed, uint64_t step, uint64_t *selected_count,
                            uint32_t nthreads)
{
    return shuffle_mt(1, params, momentum, N, P, segs, nsegs, seed, step, selected_count, nthreads);
}
