// Host-side checks of the C ABI under AddressSanitizer / UndefinedBehaviorSanitizer: every call here is
// answered on the host (argument validation, Eq. 6 helper, options, error text), so no GPU is needed.
// Built and run by tests/test_api_sanitizers.py against a build of the library whose HOST code is instrumented.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

#include "../include/wash.h"
#include "../include/wash_bench.h"

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

int main()
{
    float *fake = reinterpret_cast<float *>(uintptr_t{1} << 20);      // never dereferenced: every call below fails validation first
    float *fake2 = reinterpret_cast<float *>(uintptr_t{1} << 30);
    // Eq. 6 and its variants
    for (uint32_t L : {1u, 2u, 7u, 161u}) {
        std::vector<double> out(L);                                    // exactly L doubles
        for (int schedule = 0; schedule < 3; ++schedule) CHECK(wash_layer_probs(0.05, L, schedule, out.data()) == WASH_OK);
        CHECK(wash_layer_probs(0.05, L, 0, out.data()) == WASH_OK && out[0] == 0.05 && (L == 1 || out[L - 1] == 0.0));
    }
    double d4[4];
    CHECK(wash_layer_probs(std::nan(""), 4, 0, d4) == WASH_EINVAL);
    CHECK(wash_layer_probs(0.5, 4, 7, d4) == WASH_EINVAL);
    CHECK(wash_layer_probs(0.5, 0, 0, d4) == WASH_EINVAL);
    CHECK(wash_layer_probs(0.5, 4, 0, nullptr) == WASH_EINVAL);
    // segment validation: every list below is rejected before anything else happens
    std::vector<wash_segment> segs(300);
    for (size_t k = 0; k < segs.size(); ++k) segs[k] = wash_segment{k * 10, 10, 0.5};
    segs[299].length = 11;                                             // runs past P = 3000
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(std::strstr(wash_last_error_detail(), "299") != nullptr);
    segs[299].length = 10;
    segs[150].offset = 1495;                                           // overlaps its neighbour
    CHECK(wash_shuffle_gap(fake, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    segs[150].offset = 1500;
    segs[7].p = 1.5;
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    segs[7].p = -0.0;
    segs[8].p = std::nan("");
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    segs[8].p = 0.5;
    CHECK(wash_shuffle(fake, fake + 100, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);   // overlap
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, segs.data(), 300, 0, uint64_t{1} << 32, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle(nullptr, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle(fake, nullptr, 0, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle(fake, nullptr, WASH_MAX_N + 1, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle(fake, nullptr, 4, 0, segs.data(), 0, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    // a list of probability-zero and empty segments is valid and leaves nothing to do
    for (auto &s : segs) s.p = 0.0;
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_OK);
    CHECK(wash_shuffle_gap(fake, fake2, 4, 3000, segs.data(), 300, 0, 0, nullptr, nullptr) == WASH_OK);
    CHECK(wash_shuffle(fake, nullptr, 4, 3000, nullptr, 0, 0, 0, nullptr, nullptr) == WASH_OK);
    float *bufs[5] = {fake, fake2, fake2 + (1 << 20), fake2 + (2 << 20), fake2 + (3 << 20)};
    CHECK(wash_shuffle_states(bufs, 5, 4, 3000, segs.data(), 300, 0, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle_states(bufs, 4, 4, 3000, segs.data(), 300, 0, 0, 2, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle_states(bufs, 4, 4, 3000, segs.data(), 300, 0, 0, 1, nullptr, nullptr) == WASH_OK);
    bufs[2] = nullptr;
    CHECK(wash_shuffle_states(bufs, 4, 4, 3000, segs.data(), 300, 0, 0, 0, nullptr, nullptr) == WASH_EINVAL);
    uint64_t *word = reinterpret_cast<uint64_t *>(uintptr_t{1} << 40);
    CHECK(wash_shuffle_device_step(bufs, 2, 4, 3000, segs.data(), 300, 0, nullptr, 1, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle_device_step(bufs, 2, 4, 3000, segs.data(), 300, 0, word, 3, 0, nullptr, nullptr) == WASH_EINVAL);
    CHECK(wash_shuffle_device_step(bufs, 2, 4, 3000, segs.data(), 300, 0, word, 1, 0, word, nullptr) == WASH_EINVAL);
    // the streaming entry points
    CHECK(wash_average(nullptr, fake2, 4, 100, nullptr) == WASH_EINVAL);
    CHECK(wash_average(fake, fake + 50, 4, 100, nullptr) == WASH_EINVAL);
    CHECK(papa_ema(fake, 4, 100, INFINITY, nullptr) == WASH_EINVAL);
    CHECK(papa_ema(nullptr, 4, 100, 0.5f, nullptr) == WASH_EINVAL);
    double w[WASH_MAX_N];
    for (auto &x : w) x = 0.1;
    CHECK(wash_weighted_average(fake, nullptr, fake2, 4, 100, nullptr) == WASH_EINVAL);
    w[3] = std::nan("");
    CHECK(wash_weighted_average(fake, w, fake2, 4, 100, nullptr) == WASH_EINVAL);
    CHECK(wash_consensus_sqdist(fake, 4, 100, 50, 40, reinterpret_cast<double *>(fake2), nullptr) == WASH_EINVAL);
    CHECK(wash_consensus_sqdist_noalloc(fake, 4, 100, 50, 40, reinterpret_cast<double *>(fake2), nullptr) == WASH_EINVAL);
    CHECK(wash_consensus_sqdist_noalloc(fake, 33, 100, 0, 40, reinterpret_cast<double *>(fake2), nullptr) == WASH_EINVAL);
    CHECK(wash_set_option(WASH_OPT_SHUFFLE_BLOCKS_PER_CU, 21) == WASH_EINVAL);
    CHECK(wash_set_option(WASH_OPT_SHUFFLE_BLOCKS_PER_CU, 4) == WASH_OK);
    CHECK(wash_set_option(WASH_OPT_SHUFFLE_BLOCKS_PER_CU, 0) == WASH_OK);
    CHECK(wash_copy_f32(fake, fake + 10, 100, nullptr) == WASH_EINVAL);
    CHECK(wash_probe_scattered(fake, 3, 0, 1, 1, nullptr) == WASH_EINVAL);
    // options and texts
    CHECK(wash_set_option(WASH_OPT_TILE_COORDS, 300) == WASH_EINVAL);
    CHECK(wash_set_option(WASH_OPT_TILE_COORDS, 512) == WASH_OK && wash_set_option(WASH_OPT_TILE_COORDS, 0) == WASH_OK);
    CHECK(wash_set_option(WASH_OPT_DENSE, 3) == WASH_EINVAL && wash_set_option(WASH_OPT_DENSE, 0) == WASH_OK);
    CHECK(wash_set_option(12345, 0) == WASH_EINVAL);
    for (int status = -5; status <= 1; ++status) CHECK(wash_strerror(status) != nullptr && std::strlen(wash_strerror(status)) > 0);
    std::printf(failures ? "api sanitize driver: %d check(s) failed\n" : "api sanitize driver: all checks passed\n", failures);
    return failures ? 1 : 0;
}
