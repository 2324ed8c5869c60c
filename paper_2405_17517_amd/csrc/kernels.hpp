// Internal launchers behind the C ABI (host side; all pointers are device memory).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace wash {

// One active segment (probability > 0, length > 0) as the shuffle kernel sees it.
struct DevSegment {
    uint64_t begin;     // first coordinate
    uint64_t end;       // one past the last coordinate
    uint64_t param;     // stream v1: low 32 bits = round(p*2^32) - 1 (selected <=> mask word <= it)
                        // gap stream: bit pattern of the double 1/log2(1-p) (0.0 for p = 1)
};

constexpr uint32_t kNoSegment = 0xFFFFFFFFu;

constexpr uint32_t kMaxBufs = 4;   // parameters + up to three optimizer states

struct ShuffleArgs {
    uint32_t *bufs[kMaxBufs];   // each [N, P] as raw 32-bit words: parameters first, then optimizer states
    uint32_t nbufs;             // 1 .. kMaxBufs
    uint32_t N;
    uint64_t P;
    const DevSegment *segs;     // nsegs active segments, ascending
    uint32_t nsegs;
    const uint32_t *tile_first; // per tile: first active segment ending after the tile start, or kNoSegment
    uint64_t num_tiles;
    uint32_t tile_coords;       // stream v1: coordinates per tile (one wavefront scans one tile), multiple of 256
                                // gap stream: 1024 (a tile is one restart block; a wavefront walks `blocks_per_wave` of them)
    uint32_t blocks_per_wave;   // gap stream only: 1 .. 64
    uint32_t dense_nontemporal; // dense path only, read by the launcher: stream the rows past the caches
    uint32_t stream_stores;     // gathering kernels, read by the launchers: scattered stores are non-temporal
    uint32_t blocks_per_cu;     // read by the launchers: cap on resident blocks per compute unit (0 = none)
    uint32_t key_lo, key_hi;    // seed
    uint32_t step;              // used when step_ptr is nullptr
    const unsigned long long *step_ptr; // device step counter read by the kernel (its low 32 bits), or nullptr
    unsigned long long *step_advance;   // if set, incremented by one by the wavefront that ends the kernel (see tickets)
    unsigned long long *selected_count; // caller's counter, or nullptr
    // End-of-kernel bookkeeping (selected count, step advance) without a second launch: every active wavefront
    // adds (1 << 40 | its count) to one of kCountSlots ticket words; the wavefront that completes a word carries
    // the word's sum to the final word, and the one that completes that adds the total to the caller's counter
    // and advances the device step.  Words are zero between calls.  nullptr iff nothing was asked for.
    unsigned long long *tickets;        // kCountSlots + 1 words, one 128-byte line each (workspace of the calling stream)
    const uint32_t *expected;           // per ticket word: wavefronts that will report to it (tile kernels: active
                                        // tiles with index = word mod kCountSlots); nullptr: every wavefront of the gap grid
    uint32_t active_words;              // ticket words with expected > 0
    uint64_t nwaves;                    // gap stream: wavefronts of the grid that own at least one block
};

constexpr uint32_t kCountSlots = 256;
constexpr uint32_t kCountSlotStride = 16;   // in 8-byte words: one cache line per ticket word
constexpr size_t kTicketBytes = static_cast<size_t>(kCountSlots + 1) * kCountSlotStride * 8;
constexpr size_t kExpectedBytes = static_cast<size_t>(kCountSlots) * sizeof(uint32_t);

// a.step_advance is set only for the last kernel of a call that launches several
hipError_t launch_shuffle(const ShuffleArgs &a, hipStream_t stream);
hipError_t launch_shuffle_gap(const ShuffleArgs &a, hipStream_t stream);
// dense variant of launch_shuffle (same results): tile_coords must be 256; needs shuffle_dense_lds_bytes <= 64 KiB
size_t shuffle_dense_lds_bytes(uint32_t N, uint32_t nbufs);
hipError_t launch_shuffle_dense(const ShuffleArgs &a, hipStream_t stream);
hipError_t launch_step_advance(unsigned long long *step_advance, hipStream_t stream);   // *step_advance += 1
// chunks_per_block: 0 = choose kernel and launch shape from N and P; 1, 2, 4, 8 = the row-after-row kernel with
// that many 1024-coordinate chunks per block.  streaming: the population does not fit the Infinity Cache.
hipError_t launch_average(const float *params, float *out, uint32_t N, uint64_t P, int chunks_per_block,
                          bool streaming, hipStream_t stream);
// weights of wash_weighted_average, passed by value as a kernel argument
struct Weights {
    double w[32];
};
hipError_t launch_weighted_average(const float *params, float *out, uint32_t N, uint64_t P, const Weights &w,
                                   hipStream_t stream);

// consensus distance: `partial` is scratch of kSqdistMaxBlocks * 32 doubles
constexpr uint32_t kSqdistMaxBlocks = 4096;
constexpr size_t kSqdistScratchBytes = static_cast<size_t>(kSqdistMaxBlocks) * 32 * sizeof(double);
uint32_t sqdist_blocks(uint64_t span);
// the current device's copy of a file-scope device array of kSqdistScratchBytes (no allocation)
hipError_t static_sqdist_scratch(int device, double **out);
hipError_t launch_sqdist(const float *params, uint32_t N, uint64_t P, uint64_t g_begin, uint64_t g_end,
                         double *partial, double *out, hipStream_t stream);

hipError_t launch_scatter_probe(uint32_t *buf, uint64_t lines, int mode, uint32_t rounds, uint32_t blocks,
                                uint32_t *sink, hipStream_t stream);
// Chunks of 1024 coordinates owned by one block of the (weighted) average.  Long runs per row pay
// off once many rows are read concurrently and enough blocks remain to fill the chip (measured,
// 8 TB/s = 100 %, 1 chunk -> 8 chunks: N = 20, P = 87 M: 73 % -> 81 %; N = 10, P = 60 M: 76 -> 83;
// N = 32, P = 20 M: 77 -> 82; N = 16, P = 40 M: 76 -> 80 with 4; but N = 10, P = 26 M: 75 -> 71 and
// N = 8, P = 1.1 G: 77 -> 68).
inline int average_chunks_for(uint32_t N, uint64_t P)
{
    if (N >= 10 && P >= 40000000ull) return 8;
    if (N >= 24 && P >= 16000000ull) return 8;
    if (N >= 16 && P >= (1ull << 25)) return 4;
    return 1;
}

hipError_t launch_copy(const float *src, float *dst, uint64_t n, hipStream_t stream);
hipError_t launch_ema(float *params, uint32_t N, uint64_t P, float alpha, bool nontemporal, hipStream_t stream);

}  // namespace wash
