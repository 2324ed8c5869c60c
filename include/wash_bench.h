/*
 * wash_bench.h -- measurement aids exported by the same library as wash.h.
 * They are NOT part of the method: the benchmark uses them as yardsticks for
 * what the memory system of the chip gives a streaming pass and a scattered
 * access, and as a known-size kernel to calibrate hardware counters.
 * Conventions (device pointers, stream, status codes) are those of wash.h.
 */
#ifndef WASH_BENCH_H
#define WASH_BENCH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * dst[0..n) = src[0..n) with the same
 * 16-byte streaming access the average and the EMA use.  It reads 4n and writes
 * 4n bytes, which makes it the yardstick for the bandwidth a one-pass kernel
 * reaches on this chip and the known-size kernel that calibrates the HBM
 * traffic counters.   src, dst: device, n floats, not overlapping.
 * Errors: WASH_EINVAL for NULL pointers, n = 0, overlap.
 */
int wash_copy_f32(const float *src, float *dst, uint64_t n, void *stream);

/*
 * the yardstick for the shuffle's memory phase.
 * Every thread of `blocks` x 256 threads does `rounds` rounds of 8 independent 4-byte accesses
 * to pseudo-random 128-byte lines of buf (mode 0: loads; 1: stores; 2: a load followed by a
 * store to the same word), i.e. blocks * 256 * rounds * 8 elements per call.  Mode 3 stores whole
 * 64-byte pieces instead: four neighbouring threads write 16 bytes each to one pseudo-random
 * half line, blocks * 64 * rounds * 8 pieces per call (the memory side takes a whole piece
 * without reading it first; a 4-byte store makes it fetch the piece).  The contents of buf are
 * overwritten in modes 1 to 3.
 *   buf    device, lines * 128 bytes (16-byte aligned for mode 3)       lines  power of two, 2 .. 2^32
 * Errors: WASH_EINVAL for NULL buf, lines not a power of two, an unknown mode, rounds = 0,
 * blocks = 0 or > 2^20, a misaligned buf in mode 3.
 */
int wash_probe_scattered(float *buf, uint64_t lines, int mode, uint32_t rounds, uint32_t blocks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* WASH_BENCH_H */
