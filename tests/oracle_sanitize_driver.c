/* Exercises every entry point of the CPU oracle (oracle/wash_ref.c) on small ragged inputs in
 * exactly-sized heap buffers.  tests/test_oracle_sanitizers.py builds this file together with the
 * oracle under AddressSanitizer and UndefinedBehaviorSanitizer and runs it: an out-of-bounds access,
 * a signed overflow or a misaligned load anywhere in the oracle ends the run with an error.
 * Test infrastructure only. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint64_t offset, length; double p; } wash_ref_segment;
int wash_shuffle_ref(float *, float *, uint32_t, uint64_t, const wash_ref_segment *, uint32_t, uint64_t, uint64_t, uint64_t *);
int wash_shuffle_gap_ref(float *, float *, uint32_t, uint64_t, const wash_ref_segment *, uint32_t, uint64_t, uint64_t, uint64_t *);
int wash_shuffle_ref_window(float *, float *, uint32_t, uint64_t, uint64_t, uint64_t, uint64_t, const wash_ref_segment *,
                            uint32_t, uint64_t, uint64_t, uint64_t *);
int wash_shuffle_gap_ref_window(float *, float *, uint32_t, uint64_t, uint64_t, uint64_t, uint64_t, const wash_ref_segment *,
                                uint32_t, uint64_t, uint64_t, uint64_t *);
int wash_shuffle_ref_mt(float *, float *, uint32_t, uint64_t, const wash_ref_segment *, uint32_t, uint64_t, uint64_t,
                        uint64_t *, uint32_t);
int wash_shuffle_gap_ref_mt(float *, float *, uint32_t, uint64_t, const wash_ref_segment *, uint32_t, uint64_t, uint64_t,
                            uint64_t *, uint32_t);
int wash_ref_gap_mask(uint8_t *, uint64_t, const wash_ref_segment *, uint32_t, uint64_t, uint64_t);
int wash_average_ref(const float *, float *, uint32_t, uint64_t);
int papa_ema_ref(float *, uint32_t, uint64_t, float);
int wash_consensus_sqdist_ref(const float *, uint32_t, uint64_t, uint64_t, uint64_t, double *);
int wash_weighted_average_ref(const float *, const double *, float *, uint32_t, uint64_t);
int wash_layer_probs_ref(double, uint32_t, int, double *);
int wash_ref_permutation(uint64_t, uint64_t, uint64_t, uint32_t, uint32_t *);

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static float *population(uint32_t N, uint64_t P, uint32_t salt)
{
    float *a = (float *)malloc((size_t)N * P * sizeof(float));     /* exactly N*P elements: no slack */
    for (uint64_t k = 0; k < (uint64_t)N * P; ++k) {
        uint32_t bits = 0x3F000000u + (uint32_t)k * 7u + salt;
        memcpy(&a[k], &bits, 4);
    }
    return a;
}

/* XOR of all N*P bit patterns: unchanged by any permutation of values */
static uint32_t fingerprint(const float *a, uint64_t count)
{
    uint32_t x = 0, b;
    for (uint64_t k = 0; k < count; ++k) { memcpy(&b, &a[k], 4); x ^= b; }
    return x;
}

static void one_shape(uint32_t N, uint64_t P)
{
    wash_ref_segment segs[5];
    uint32_t nsegs = 0;
    if (P >= 40) {
        segs[nsegs++] = (wash_ref_segment){0, P / 4, 0.5};
        segs[nsegs++] = (wash_ref_segment){P / 4, 0, 0.9};            /* empty */
        segs[nsegs++] = (wash_ref_segment){P / 4 + 3, P / 2 - P / 4 - 3, 1.0};
        segs[nsegs++] = (wash_ref_segment){P / 2, P - P / 2 - 1, 0.01};
        segs[nsegs++] = (wash_ref_segment){P - 1, 1, 1.0};            /* last coordinate */
    } else {
        segs[nsegs++] = (wash_ref_segment){0, P, 0.7};
    }
    const uint64_t seed = 0xFEDCBA9876543210ull, step = 4294967295ull;
    for (int gap = 0; gap < 2; ++gap) {
        float *a = population(N, P, 1), *m = population(N, P, 2), *b = population(N, P, 1), *bm = population(N, P, 2);
        const uint32_t fa = fingerprint(a, (uint64_t)N * P), fm = fingerprint(m, (uint64_t)N * P);
        uint64_t c1 = 0, c2 = 0, c3 = 0;
        CHECK((gap ? wash_shuffle_gap_ref : wash_shuffle_ref)(a, m, N, P, segs, nsegs, seed, step, &c1) == 0);
        CHECK((gap ? wash_shuffle_gap_ref_mt : wash_shuffle_ref_mt)(b, bm, N, P, segs, nsegs, seed, step, &c2, 3) == 0);
        CHECK(c1 == c2 && memcmp(a, b, (size_t)N * P * 4) == 0 && memcmp(m, bm, (size_t)N * P * 4) == 0);
        CHECK(fingerprint(a, (uint64_t)N * P) == fa && fingerprint(m, (uint64_t)N * P) == fm);
        /* the last window of the row, in a buffer of exactly its size */
        const uint64_t g0 = gap ? (P / 1024) * 1024 : P - (P < 37 ? P : 37);
        if (g0 < P) {
            const uint64_t W = P - g0;
            float *w = (float *)malloc((size_t)N * W * 4), *ref = population(N, P, 1);
            for (uint32_t n = 0; n < N; ++n) memcpy(w + n * W, ref + n * P + g0, (size_t)W * 4);
            CHECK((gap ? wash_shuffle_gap_ref_window : wash_shuffle_ref_window)(w, NULL, N, P, W, g0, P, segs, nsegs, seed,
                                                                               step, &c3) == 0);
            for (uint32_t n = 0; n < N; ++n) CHECK(memcmp(w + n * W, a + n * P + g0, (size_t)W * 4) == 0);
            free(w); free(ref);
        }
        if (gap) {
            uint8_t *mask = (uint8_t *)calloc(P, 1);
            CHECK(wash_ref_gap_mask(mask, P, segs, nsegs, seed, step) == 0);
            uint64_t ones = 0;
            for (uint64_t g = 0; g < P; ++g) ones += mask[g];
            CHECK(ones == c1);
            free(mask);
        }
        free(a); free(m); free(b); free(bm);
    }
    float *a = population(N, P, 5), *out = (float *)malloc(P * 4), *out2 = (float *)malloc(P * 4);
    double w[32], d[32], total = 0.0;
    for (uint32_t n = 0; n < N; ++n) w[n] = 1.0 / N;
    CHECK(wash_average_ref(a, out, N, P) == 0);
    CHECK(wash_weighted_average_ref(a, w, out2, N, P) == 0);
    CHECK(wash_consensus_sqdist_ref(a, N, P, 0, P, d) == 0);
    CHECK(wash_consensus_sqdist_ref(a, N, P, P - 1, P, d) == 0);
    CHECK(papa_ema_ref(a, N, P, 0.0f) == 0);                        /* every row becomes the average */
    for (uint32_t n = 0; n < N; ++n) CHECK(memcmp(a + n * P, out, (size_t)P * 4) == 0);
    CHECK(wash_consensus_sqdist_ref(a, N, P, 0, P, d) == 0);
    for (uint32_t n = 0; n < N; ++n) total += d[n];
    CHECK(total == 0.0);
    free(a); free(out); free(out2);
}

int main(void)
{
    const uint32_t Ns[] = {1, 2, 5, 20, 32};
    const uint64_t Ps[] = {1, 3, 39, 40, 1023, 1024, 1025, 5000};
    for (unsigned i = 0; i < sizeof(Ns) / sizeof(Ns[0]); ++i)
        for (unsigned j = 0; j < sizeof(Ps) / sizeof(Ps[0]); ++j) one_shape(Ns[i], Ps[j]);
    double probs[7];
    for (int schedule = 0; schedule < 3; ++schedule) CHECK(wash_layer_probs_ref(0.3, 7, schedule, probs) == 0);
    CHECK(wash_layer_probs_ref(0.3, 1, 0, probs) == 0 && probs[0] == 0.3);
    uint32_t perm[32];
    CHECK(wash_ref_permutation(1, 2, (1ull << 40) - 1, 32, perm) == 0);
    /* invalid arguments come back as errors, not as accesses */
    float one = 1.0f;
    wash_ref_segment bad = {5, 10, 0.5};
    CHECK(wash_shuffle_ref(&one, NULL, 1, 1, &bad, 1, 0, 0, NULL) != 0);
    CHECK(wash_shuffle_ref(&one, NULL, 33, 1, NULL, 0, 0, 0, NULL) != 0);
    CHECK(wash_shuffle_gap_ref(&one, NULL, 1, 1, &bad, 1, 0, 0, NULL) != 0);
    printf(failures ? "sanitize driver: %d check(s) failed\n" : "sanitize driver: all checks passed\n", failures);
    return failures ? 1 : 0;
}
