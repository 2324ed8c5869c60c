// wash_shuffle kernels for gfx950: the shuffling step of WASH (Sec. 3, Eq. 3;
// Alg. 1, shuffling step), with the optimizer state(s) moved along (WASH+Opt).
// Three kernels: shuffle_kernel (default stream, sparse: gathers single values),
// shuffle_dense_kernel (default stream, p >= 0.08: streams whole strips through
// LDS; same bits) and shuffle_gap_kernel (gap-sampled mask stream).
//
// shuffle_kernel: one wavefront owns one tile of consecutive coordinates and
// works alone (no workgroup barrier anywhere):
//   scan     each lane draws the mask words of 4 consecutive coordinates with
//            one Philox call and compares them with the segment threshold;
//            the Bernoulli mask is never written to memory.
//   compact  selected coordinates are appended to a small per-wave LDS queue
//            through ballot + lane-prefix counts, so the expensive part below
//            runs on dense lanes and HBM traffic follows p*N*P, not N*P.
//   permute  whenever 64 coordinates are queued (and once at the end) each
//            lane takes one coordinate: its N values (and N momentum values)
//            are gathered into an LDS slab [N][64] by direct global-to-LDS
//            loads (all N in flight, no register array), the descending
//            Fisher-Yates walk swaps slab rows in place, and because slot i is
//            final after step i its value is stored to row i right there.
// Everything random is integer arithmetic, so the result is bit-identical to
// any other implementation of the same stream.
#include "gaplog.hpp"
#include "kernels.hpp"
#include "philox.hpp"

namespace wash {

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr uint32_t kMaxCalls = 8;       // Philox calls for the N-1 <= 31 permutation words of a coordinate
constexpr int kQueueCap = 64 + 256;   // a batch is cut as soon as 64 are queued; one scan adds <= 256

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

// Order LDS traffic between lanes of one wavefront (no instruction is emitted:
// a wavefront's LDS operations execute in issue order).
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The step of this launch: a kernel argument, or the low 32 bits of a device counter (so that a
// captured launch can be replayed with a step that advances).
__device__ __forceinline__ uint32_t step_of(const ShuffleArgs &a)
{
    return a.step_ptr != nullptr ? static_cast<uint32_t>(*a.step_ptr) : a.step;
}

// Called once by every wavefront that `expected` counts, at its end (lane 0 acts): see ShuffleArgs::tickets.
__device__ __forceinline__ void report_wave(const ShuffleArgs &a, uint64_t index, uint32_t selected)
{
    if (a.tickets == nullptr || lane_id() != 0) return;
    const uint32_t word = static_cast<uint32_t>(index % kCountSlots);
    const uint64_t expected = a.expected != nullptr ? a.expected[word]
                                                    : a.nwaves / kCountSlots + (word < a.nwaves % kCountSlots ? 1u : 0u);
    constexpr unsigned long long kOne = 1ull << 40, kSum = kOne - 1;      // a word sums at most P / 256 < 2^40
    unsigned long long *slot = a.tickets + word * kCountSlotStride;
    const unsigned long long now = atomicAdd(slot, kOne | selected) + (kOne | selected);
    if ((now >> 40) != expected) return;
    *slot = 0;                                                           // nobody else comes to this word in this kernel
    constexpr unsigned long long kOne2 = 1ull << 48, kSum2 = kOne2 - 1;   // the total is at most P <= 2^40
    unsigned long long *last = a.tickets + kCountSlots * kCountSlotStride;
    const unsigned long long mine = kOne2 | (now & kSum);
    const unsigned long long all = atomicAdd(last, mine) + mine;
    if ((all >> 48) != a.active_words) return;
    *last = 0;
    if (a.selected_count != nullptr && (all & kSum2) != 0) atomicAdd(a.selected_count, all & kSum2);
    if (a.step_advance != nullptr) *a.step_advance += 1;                  // every wavefront has read the step by now
}

typedef __attribute__((address_space(1))) const void *global_cptr;
typedef __attribute__((address_space(3))) void *lds_ptr;

// One dword per active lane straight from global memory into LDS at row[lane]
// (no VGPR in between): the N gathers of a batch are all in flight at once
// whatever N is, and the slab is filled without a register array.
__device__ __forceinline__ void gather_row_to_lds(const uint32_t *src, uint32_t *row)
{
    __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)row, 4, 0, 0);
}

// The same for data that is read once and written once (the dense path): non-temporal, like the
// streaming kernels of this library.
__device__ __forceinline__ void stream_row_to_lds(const uint32_t *src, uint32_t *row)
{
    __builtin_amdgcn_global_load_lds((global_cptr)src, (lds_ptr)row, 4, 0, 2);   // aux bit 1: nt
}

// The swap partners j_i of the descending Fisher-Yates walk of coordinate g (i = N-1 .. 1,
// j_i = (w * (i+1)) >> 32 with the permutation words w of the stream, four per Philox call), packed
// one byte each, four to a register.  The packs sit in a register ring that is rotated instead of
// indexed, so the loops stay rolled: after the kMaxCalls rotations below the pack of call c is in ring[c].
__device__ __forceinline__ void draw_swap_partners(const ShuffleArgs &a, uint32_t step, uint64_t g,
                                                   uint32_t (&ring)[kMaxCalls])
{
    const uint32_t N = a.N;
    const uint32_t g_lo = static_cast<uint32_t>(g), g_hi = static_cast<uint32_t>(g >> 32);
    const uint32_t nswaps = N - 1;
    const uint32_t ncalls = (nswaps + 3u) / 4u;             // <= kMaxCalls
#pragma unroll
    for (uint32_t q = 0; q < kMaxCalls; ++q) ring[q] = 0;
#pragma unroll 1
    for (uint32_t call = 0; call < kMaxCalls; ++call) {
        uint32_t pack = 0;
        if (call < ncalls) {
            const Words4 r = philox4x32_10(g_lo, g_hi, step, 1u + call, a.key_lo, a.key_hi);
            const uint32_t w[4] = {r.w0, r.w1, r.w2, r.w3};
#pragma unroll
            for (uint32_t k = 0; k < 4; ++k) {
                const uint32_t t = call * 4u + k;
                if (t < nswaps) pack |= __umulhi(w[k], N - t) << (8u * k);   // i + 1 = N - t
            }
        }
#pragma unroll
        for (uint32_t q = 0; q + 1 < kMaxCalls; ++q) ring[q] = ring[q + 1];
        ring[kMaxCalls - 1] = pack;
    }
}

// Gather, permute and scatter up to 64 queued coordinates, one per lane.
// kBufs buffers (the parameters, then the optimizer states) share the mask and the permutation;
// buffer b uses the slab at slab + b * N * 64.
// kStream: the scattered stores are non-temporal.  Request sizes and HBM bytes stay what they are (measured:
// 81 bytes fetched and 25 bytes written per moved value with any of sc0 / sc1 / nt on the gathers or the stores),
// but on populations far beyond the caches the kernel gains 3 % (N = 8, P = 1.1e9, two buffers: 14.65 -> 14.16 ms;
// no change at 2 GB).  Non-temporal gathers lose 35-45 % and are not used.
template <int kBufs, bool kStream, typename QueueEntry>
__device__ __forceinline__ void permute_batch(const ShuffleArgs &a, uint32_t step, uint64_t tile_begin,
                                              const QueueEntry *queue, uint32_t nbatch, uint32_t *slab)
{
    const uint32_t lane = lane_id();
    if (lane >= nbatch) return;
    const uint64_t g = tile_begin + queue[lane];
    const uint32_t N = a.N;
    const uint64_t P = a.P;
    const uint32_t slab_words = N * kWave;
    uint32_t *col[kBufs];
#pragma unroll
    for (int b = 0; b < kBufs; ++b) col[b] = a.bufs[b] + g;

    // gather the column(s) into the slab(s): slab[b][n][lane]
    for (uint32_t n = 0; n < N; ++n) {
#pragma unroll
        for (int b = 0; b < kBufs; ++b)
            gather_row_to_lds(col[b] + static_cast<uint64_t>(n) * P, slab + b * slab_words + n * kWave);
    }
    // While the gathers are in flight, draw the swap partners: they depend on the coordinate only.
    const uint32_t nswaps = N - 1;
    const uint32_t ncalls = (nswaps + 3u) / 4u;             // <= kMaxCalls
    uint32_t ring[kMaxCalls];
    draw_swap_partners(a, step, g, ring);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // The walk is applied to the values themselves: swapping slab rows i and j keeps
    // slab[n] == old[perm[n]]; row i is final after step i and goes straight to memory.
    // A row that keeps its own value (a fixed point of the permutation: one per coordinate on
    // average) is not written: `moved` has bit k set once slot k holds a value from another row.
    uint32_t moved = 0;
    uint32_t i = nswaps;
    for (uint32_t call = 0; call < ncalls; ++call) {
        const uint32_t pack = ring[0];
#pragma unroll
        for (uint32_t q = 0; q + 1 < kMaxCalls; ++q) ring[q] = ring[q + 1];
#pragma unroll
        for (uint32_t k = 0; k < 4; ++k) {
            if (i == 0) break;
            const uint32_t j = (pack >> (8u * k)) & 0xFFu;
            const bool write_row = (j != i) || ((moved >> i) & 1u);
#pragma unroll
            for (int b = 0; b < kBufs; ++b) {
                uint32_t *sl = slab + b * slab_words;
                const uint32_t vi = sl[i * kWave + lane];
                const uint32_t vj = sl[j * kWave + lane];
                if (write_row) {
                    if (kStream) __builtin_nontemporal_store(vj, &col[b][static_cast<uint64_t>(i) * P]);
                    else col[b][static_cast<uint64_t>(i) * P] = vj;
                }
                sl[j * kWave + lane] = vi;
            }
            if (j != i) moved |= 1u << j;
            --i;
        }
    }
    if (moved & 1u) {
#pragma unroll
        for (int b = 0; b < kBufs; ++b) {
            if (kStream) __builtin_nontemporal_store(slab[b * slab_words + lane], &col[b][0]);
            else col[b][0] = slab[b * slab_words + lane];
        }
    }
}

// The Bernoulli mask (Eq. 3) of the four coordinates 4*quad .. 4*quad+3: one Philox call, the four
// words compared with the thresholds of the segments the coordinates lie in.  `uniform`: the whole
// tile lies in segment seg0.  Otherwise `walk` is the lane's cursor into the segment table; the
// coordinates of a lane only grow from call to call, so the cursor only moves forward.
__device__ __forceinline__ void select_quad(const ShuffleArgs &a, uint32_t step, uint64_t quad, uint64_t tile_end,
                                            bool uniform, const DevSegment &seg0, uint32_t &walk, bool (&sel)[4])
{
    const uint64_t g0 = quad << 2;
    const Words4 r = philox4x32_10(static_cast<uint32_t>(quad), static_cast<uint32_t>(quad >> 32),
                                   step, 0u, a.key_lo, a.key_hi);
    const uint32_t w[4] = {r.w0, r.w1, r.w2, r.w3};
    if (uniform) {
#pragma unroll
        for (int k = 0; k < 4; ++k) sel[k] = (w[k] <= static_cast<uint32_t>(seg0.param)) && (g0 + k < tile_end);
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t g = g0 + k;
            while (walk < a.nsegs && a.segs[walk].end <= g) ++walk;
            bool s = false;
            if (walk < a.nsegs && g < tile_end) {
                const DevSegment sg = a.segs[walk];
                s = (sg.begin <= g) && (w[k] <= static_cast<uint32_t>(sg.param));
            }
            sel[k] = s;
        }
    }
}

template <int kBufs, bool kStream>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void shuffle_kernel(const ShuffleArgs a)
{
    extern __shared__ uint32_t lds[];
    const uint32_t lane = lane_id();
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t waves_per_block = blockDim.x / kWave;
    const uint64_t tile = static_cast<uint64_t>(blockIdx.x) * waves_per_block + wave_in_block;
    if (tile >= a.num_tiles) return;
    const uint32_t first = a.tile_first[tile];
    if (first == kNoSegment) return;
    const uint32_t step = step_of(a);

    const uint32_t slab_words = a.N * kWave;
    // per wave: [queue: 320 x u16 (tile offsets; a tile has at most 65536 coordinates)][slab(s)]
    const uint32_t per_wave = kQueueCap / 2 + slab_words * kBufs;
    uint32_t *base = lds + wave_in_block * per_wave;
    uint16_t *queue = reinterpret_cast<uint16_t *>(base);
    uint32_t *slab = base + kQueueCap / 2;

    const uint64_t tile_begin = tile * a.tile_coords;
    const uint64_t tile_end = min(tile_begin + a.tile_coords, a.P);
    const DevSegment seg0 = a.segs[first];
    const bool uniform = seg0.begin <= tile_begin && seg0.end >= tile_end;
    const uint32_t iters = static_cast<uint32_t>((tile_end - tile_begin + 255u) / 256u);

    uint32_t queued = 0;      // wave-uniform
    uint32_t selected = 0;    // wave-uniform, total of the tile
    uint32_t walk = first;    // per lane: segment cursor for tiles that straddle segments

    for (uint32_t it = 0; it < iters; ++it) {
        const uint64_t quad = (tile_begin >> 2) + static_cast<uint64_t>(it) * kWave + lane;
        const uint64_t g0 = quad << 2;
        bool sel[4];
        select_quad(a, step, quad, tile_end, uniform, seg0, walk, sel);
        if (__ballot(sel[0] | sel[1] | sel[2] | sel[3]) == 0) continue;

        // append in ascending coordinate order (lane-major, then k), so that neighbours in the
        // queue are neighbours in memory and a batch touches as few cache lines as possible
        const uint64_t b0 = __ballot(sel[0]), b1 = __ballot(sel[1]), b2 = __ballot(sel[2]), b3 = __ballot(sel[3]);
        uint32_t pos = queued + lanes_below(b0) + lanes_below(b1) + lanes_below(b2) + lanes_below(b3);
        const uint32_t off0 = static_cast<uint32_t>(g0 - tile_begin);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (sel[k]) queue[pos++] = static_cast<uint16_t>(off0 + k);
        }
        queued += __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3);
        while (queued >= kWave) {
            wave_lds_sync();
            permute_batch<kBufs, kStream>(a, step, tile_begin, queue + (queued - kWave), kWave, slab);
            queued -= kWave;
            selected += kWave;
            wave_lds_sync();
        }
    }
    if (queued > 0) {
        wave_lds_sync();
        permute_batch<kBufs, kStream>(a, step, tile_begin, queue, queued, slab);
        selected += queued;
    }
    // One atomic per wavefront on a single address would serialise the whole grid at the memory side
    // (measured: 92 us instead of 14 on 2728 wavefronts); the reports are spread over kCountSlots cache lines.
    report_wave(a, tile, selected);
}

// ---------------------------------------------------------------------------------------------
// Dense variant of the same stream for high probabilities.  Once most 64-byte half lines of a row
// hold a selected coordinate, scattered 4-byte accesses cost more than streaming the rows through
// LDS: one wavefront (one workgroup) owns one strip of 256 coordinates, loads it from all N rows
// of every buffer with coalesced global->LDS loads, permutes the selected columns in LDS (the same
// mask, the same swap partners, hence the same bits as shuffle_kernel) and writes the rows back
// with 16-byte stores.  Unselected coordinates of the strip are rewritten with their own values.
constexpr uint32_t kStrip = 256;
constexpr uint32_t kXcds = 8;
typedef uint32_t u4u __attribute__((ext_vector_type(4), aligned(4)));   // rows are only 4-byte aligned

template <int kBufs, bool kStream>
__global__ __launch_bounds__(kWave) void shuffle_dense_kernel(const ShuffleArgs a)
{
    extern __shared__ uint32_t lds[];
    const uint32_t lane = lane_id();
    // Workgroups are handed to the 8 XCDs round robin, and each XCD has its own L2.  Give every XCD one
    // contiguous run of strips, so that the cache line two neighbouring strips share when rows are not
    // 128-byte aligned is fetched into one L2 only.
    const uint64_t per_xcd = (a.num_tiles + kXcds - 1) / kXcds;
    const uint64_t tile = (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (tile >= a.num_tiles) return;
    const uint32_t first = a.tile_first[tile];
    if (first == kNoSegment) return;
    const uint32_t step = step_of(a);
    const uint32_t N = a.N;
    const uint64_t P = a.P;
    const uint64_t begin = tile * kStrip;
    const uint64_t end = min(begin + kStrip, P);
    const DevSegment seg0 = a.segs[first];
    const bool uniform = seg0.begin <= begin && seg0.end >= end;

    uint32_t walk = first;
    bool sel[4];
    select_quad(a, step, (begin >> 2) + lane, end, uniform, seg0, walk, sel);
    const uint64_t b0 = __ballot(sel[0]), b1 = __ballot(sel[1]), b2 = __ballot(sel[2]), b3 = __ballot(sel[3]);
    const uint32_t count = __popcll(b0) + __popcll(b1) + __popcll(b2) + __popcll(b3);
    if (count == 0) {
        report_wave(a, tile, 0);
        return;
    }

    // [selected offsets: 256 x u16][slab: kBufs x N rows x 256 coordinates]
    uint16_t *picked = reinterpret_cast<uint16_t *>(lds);
    uint32_t *slab = lds + kStrip / 2;
    const uint32_t width = static_cast<uint32_t>(end - begin);      // 1 .. 256
    // kStream: non-temporal loads and stores.  Together they pay off on large populations (measured, both
    // or neither: N = 20, P = 87 M: 3.15 -> 2.92 ms; N = 10, P = 26 M, two buffers: 0.86 -> 0.89 ms; one of
    // the two alone is slower everywhere, 3.70 ms with the loads alone).  A template parameter and not a
    // run-time flag: the two stores of a run-time branch are merged into one plain store.
    constexpr bool nt = kStream;

    // rows -> LDS: four loads of 64 consecutive words per row, lane l of load q brings coordinate 64 q + l
    for (uint32_t n = 0; n < N; ++n) {
#pragma unroll
        for (int b = 0; b < kBufs; ++b) {
            const uint32_t *row = a.bufs[b] + static_cast<uint64_t>(n) * P + begin;
            uint32_t *dst = slab + (b * N + n) * kStrip;
#pragma unroll
            for (uint32_t q = 0; q < kStrip / kWave; ++q)
                if (q * kWave + lane < width) {
                    if (nt) stream_row_to_lds(row + q * kWave + lane, dst + q * kWave);
                    else gather_row_to_lds(row + q * kWave + lane, dst + q * kWave);
                }
        }
    }
    // meanwhile: the selected offsets, ascending
    uint32_t pos = lanes_below(b0) + lanes_below(b1) + lanes_below(b2) + lanes_below(b3);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        if (sel[k]) picked[pos++] = static_cast<uint16_t>(4u * lane + k);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    wave_lds_sync();

    const uint32_t nswaps = N - 1;
    const uint32_t ncalls = (nswaps + 3u) / 4u;
    for (uint32_t done = 0; done < count; done += kWave) {
        if (done + lane < count) {
            const uint32_t c = picked[done + lane];
            uint32_t ring[kMaxCalls];
            draw_swap_partners(a, step, begin + c, ring);
            uint32_t i = nswaps;
            for (uint32_t call = 0; call < ncalls; ++call) {
                const uint32_t pack = ring[0];
#pragma unroll
                for (uint32_t q = 0; q + 1 < kMaxCalls; ++q) ring[q] = ring[q + 1];
#pragma unroll
                for (uint32_t k = 0; k < 4; ++k) {
                    if (i == 0) break;
                    const uint32_t j = (pack >> (8u * k)) & 0xFFu;
#pragma unroll
                    for (int b = 0; b < kBufs; ++b) {
                        uint32_t *colm = slab + b * N * kStrip + c;
                        const uint32_t vi = colm[i * kStrip];
                        const uint32_t vj = colm[j * kStrip];
                        colm[i * kStrip] = vj;
                        colm[j * kStrip] = vi;
                    }
                    --i;
                }
            }
        }
    }
    wave_lds_sync();

    // LDS -> rows: 16 bytes per lane (word by word in a ragged last strip)
    const uint32_t c0 = 4u * lane;
    for (uint32_t n = 0; n < N; ++n) {
#pragma unroll
        for (int b = 0; b < kBufs; ++b) {
            uint32_t *row = a.bufs[b] + static_cast<uint64_t>(n) * P + begin;
            const uint32_t *src = slab + (b * N + n) * kStrip + c0;
            if (c0 + 4u <= width) {
                const u4u v = {src[0], src[1], src[2], src[3]};
                if (nt) __builtin_nontemporal_store(v, reinterpret_cast<u4u *>(row + c0));
                else *reinterpret_cast<u4u *>(row + c0) = v;
            } else {
                for (uint32_t k = 0; c0 + k < width; ++k) row[c0 + k] = src[k];
            }
        }
    }
    report_wave(a, tile, count);
}

// A call with nothing to shuffle still advances the device step counter.
__global__ void step_advance_kernel(unsigned long long *step_advance)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *step_advance += 1;
}


// ---------------------------------------------------------------------------------------------
// Gap stream: the mask is walked, not scanned.  A lane owns one restart block of 1024
// coordinates and draws the distances between selected coordinates (geometric by inversion), so
// the random-number work follows p*P instead of P.  A wavefront walks `blocks_per_wave`
// neighbouring blocks in lock step; every lane parks its finds in a short private list, and when
// a list fills up (or every lane is done) the lists are poured, lane after lane, into the queue:
// that keeps the queue in ascending coordinate order, so the permute batches touch neighbouring
// cache lines exactly as in the scanning kernel.

constexpr uint32_t kGapQueueCap = 512;       // finds a wavefront can park between two flushes, shared by its lanes

template <int kBufs, bool kStream>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void shuffle_gap_kernel(const ShuffleArgs a)
{
    extern __shared__ uint32_t lds[];
    const uint32_t lane = lane_id();
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint32_t waves_per_block = blockDim.x / kWave;
    const uint64_t wave = static_cast<uint64_t>(blockIdx.x) * waves_per_block + wave_in_block;
    const uint32_t bpw = a.blocks_per_wave;
    const uint64_t first_block = wave * bpw;
    if (first_block >= a.num_tiles) return;
    const uint32_t step = step_of(a);

    // per wave: [queue: 512 x u16][lists: 512 x u16][slab(s)]; a lane's list holds 512 / blocks_per_wave finds
    const uint32_t list_cap = kGapQueueCap / bpw;
    const uint32_t slab_words = a.N * kWave;
    const uint32_t per_wave = kGapQueueCap + slab_words * kBufs;
    uint32_t *base = lds + wave_in_block * per_wave;
    uint16_t *queue = reinterpret_cast<uint16_t *>(base);
    uint16_t *list = queue + kGapQueueCap + lane * list_cap;
    uint32_t *slab = base + kGapQueueCap;
    const uint64_t tile_begin = first_block * kGapPiece;

    // lane state: the piece [piece_off .. end_off) of its block it is walking, as offsets in the block
    const uint64_t blk = first_block + lane;
    const uint64_t blk_begin = blk * kGapPiece;
    const uint64_t blk_end = min(blk_begin + kGapPiece, a.P);
    bool active = false;
    uint32_t seg = kNoSegment, piece_off = 0, end_off = 0, next_off = 0, draw = 0;
    double scale = 0.0;
    if (lane < bpw && blk < a.num_tiles) {
        seg = a.tile_first[blk];
        active = seg != kNoSegment;
    }
    if (active) {
        const DevSegment sg = a.segs[seg];
        piece_off = static_cast<uint32_t>(max(sg.begin, blk_begin) - blk_begin);
        end_off = static_cast<uint32_t>(min(sg.end, blk_end) - blk_begin);
        scale = __longlong_as_double(static_cast<long long>(sg.param));
        next_off = piece_off;
    }

    uint32_t parked = 0;       // finds in this lane's list
    uint32_t selected = 0;     // wave-uniform, total of the wave
    Words4 r{0, 0, 0, 0};
    while (__ballot(active) != 0) {
        if (active) {
            if ((draw & 1u) == 0) {
                const uint64_t s = blk_begin + piece_off;
                r = philox4x32_10(static_cast<uint32_t>(s), static_cast<uint32_t>(s >> 32), step,
                                  0x80000000u + (draw >> 1), a.key_lo, a.key_hi);
            }
            const uint32_t hi = (draw & 1u) ? r.w2 : r.w0, lo = (draw & 1u) ? r.w3 : r.w1;
            const uint64_t U = ((static_cast<uint64_t>(hi) << 32) | lo) >> 11;
            const uint32_t found = next_off + gap_distance(U, scale) - 1u;
            if (found < end_off) {
                list[parked++] = static_cast<uint16_t>(found);
                next_off = found + 1u;
                ++draw;
            } else {
                // this piece is finished: the next segment may start inside the same block
                ++seg;
                active = false;
                if (seg < a.nsegs) {
                    const DevSegment sg = a.segs[seg];
                    if (sg.begin < blk_end) {
                        piece_off = static_cast<uint32_t>(sg.begin - blk_begin);
                        end_off = static_cast<uint32_t>(min(sg.end, blk_end) - blk_begin);
                        scale = __longlong_as_double(static_cast<long long>(sg.param));
                        next_off = piece_off;
                        draw = 0;
                        active = true;
                    }
                }
            }
        }
        // pour the lists into the queue when one is full or everybody is done
        if (__ballot(parked == list_cap) == 0 && __ballot(active) != 0) continue;
        uint32_t before = parked;                    // exclusive prefix of `parked` over the lanes
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t up = __shfl_up(before, off, kWave);
            if (lane >= static_cast<uint32_t>(off)) before += up;
        }
        const uint32_t total = __shfl(before, kWave - 1, kWave);
        before -= parked;
        for (uint32_t j = 0; j < parked; ++j) queue[before + j] = static_cast<uint16_t>(lane * kGapPiece + list[j]);
        parked = 0;
        wave_lds_sync();
        for (uint32_t done = 0; done < total; done += kWave) {
            permute_batch<kBufs, kStream>(a, step, tile_begin, queue + done, min(total - done, static_cast<uint32_t>(kWave)), slab);
        }
        selected += total;
        wave_lds_sync();
    }
    report_wave(a, wave, selected);
}

}  // namespace

// Dynamic LDS a block asks for beyond what it uses, so that at most `blocks_per_cu` blocks share the 160 KB of a
// compute unit (0: no cap).  `used` is what the kernel itself needs.
static size_t lds_with_cap(size_t used, uint32_t blocks_per_cu)
{
    if (blocks_per_cu == 0 || blocks_per_cu > 20) return used;
    const size_t want = (160u * 1024u - 1024u) / blocks_per_cu / 256u * 256u;
    return want > used ? want : used;
}

template <auto Kernel>
static hipError_t allow_large_lds()
{
    static bool done[64] = {};
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= 64) return hipErrorInvalidDevice;
    if (done[device]) return hipSuccess;          // callers hold the library mutex
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            159 * 1024);
    if (e == hipSuccess) done[device] = true;
    return e;
}

hipError_t launch_step_advance(unsigned long long *step_advance, hipStream_t stream)
{
    hipLaunchKernelGGL(step_advance_kernel, dim3(1), dim3(kWave), 0, stream, step_advance);
    return hipGetLastError();
}

// a kernel with nothing to do: only the step advance is left of the call
static hipError_t nothing_to_launch(const ShuffleArgs &a, hipStream_t stream)
{
    return a.step_advance != nullptr ? launch_step_advance(a.step_advance, stream) : hipSuccess;
}

hipError_t launch_shuffle(const ShuffleArgs &a, hipStream_t stream)
{
    if (a.num_tiles == 0 || a.nsegs == 0) return nothing_to_launch(a, stream);
    // the direct-to-LDS loads address LDS through a 16-bit offset: keep a block's partition below 64 KiB
    if (a.nbufs == 0 || a.nbufs > kMaxBufs) return hipErrorInvalidValue;
    if (a.tickets != nullptr && a.expected == nullptr) return hipErrorInvalidValue;
    const size_t per_wave = (kQueueCap / 2 + static_cast<size_t>(a.N) * kWave * a.nbufs) * sizeof(uint32_t);
    uint32_t waves = kWavesPerBlock;
    while (waves > 1 && per_wave * waves > 65536) waves >>= 1;
    if (per_wave * waves > 65536) return hipErrorInvalidConfiguration;
    const uint64_t blocks64 = (a.num_tiles + waves - 1) / waves;
    if (blocks64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    const dim3 grid(static_cast<uint32_t>(blocks64)), block(kWave * waves);
    const size_t lds_bytes = lds_with_cap(per_wave * waves, a.blocks_per_cu);
    hipError_t ea = hipSuccess;
#define WASH_LAUNCH_SPARSE(B, S)                                                                                   \
    do {                                                                                                           \
        if (lds_bytes > 65536) ea = allow_large_lds<shuffle_kernel<B, S>>();                                       \
        if (ea == hipSuccess) hipLaunchKernelGGL((shuffle_kernel<B, S>), grid, block, lds_bytes, stream, a);      \
    } while (0)
    if (a.stream_stores) {
        switch (a.nbufs) {
        case 1: WASH_LAUNCH_SPARSE(1, true); break;
        case 2: WASH_LAUNCH_SPARSE(2, true); break;
        case 3: WASH_LAUNCH_SPARSE(3, true); break;
        default: WASH_LAUNCH_SPARSE(4, true); break;
        }
    } else {
        switch (a.nbufs) {
        case 1: WASH_LAUNCH_SPARSE(1, false); break;
        case 2: WASH_LAUNCH_SPARSE(2, false); break;
        case 3: WASH_LAUNCH_SPARSE(3, false); break;
        default: WASH_LAUNCH_SPARSE(4, false); break;
        }
    }
#undef WASH_LAUNCH_SPARSE
    if (ea != hipSuccess) return ea;
    return hipGetLastError();
}

size_t shuffle_dense_lds_bytes(uint32_t N, uint32_t nbufs)
{
    return (kStrip / 2 + static_cast<size_t>(N) * nbufs * kStrip) * sizeof(uint32_t);
}

hipError_t launch_shuffle_dense(const ShuffleArgs &a, hipStream_t stream)
{
    if (a.num_tiles == 0 || a.nsegs == 0) return nothing_to_launch(a, stream);
    if (a.nbufs == 0 || a.nbufs > kMaxBufs || a.tile_coords != kStrip) return hipErrorInvalidValue;
    if (a.tickets != nullptr && a.expected == nullptr) return hipErrorInvalidValue;
    const size_t lds_bytes = shuffle_dense_lds_bytes(a.N, a.nbufs);
    // the direct-to-LDS loads address LDS through a 16-bit offset
    if (lds_bytes > 65536 || a.num_tiles > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    const uint64_t blocks64 = (a.num_tiles + kXcds - 1) / kXcds * kXcds;
    if (blocks64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    const dim3 grid(static_cast<uint32_t>(blocks64)), block(kWave);
    if (a.dense_nontemporal) {
        switch (a.nbufs) {
        case 1: hipLaunchKernelGGL((shuffle_dense_kernel<1, true>), grid, block, lds_bytes, stream, a); break;
        case 2: hipLaunchKernelGGL((shuffle_dense_kernel<2, true>), grid, block, lds_bytes, stream, a); break;
        case 3: hipLaunchKernelGGL((shuffle_dense_kernel<3, true>), grid, block, lds_bytes, stream, a); break;
        default: hipLaunchKernelGGL((shuffle_dense_kernel<4, true>), grid, block, lds_bytes, stream, a); break;
        }
    } else {
        switch (a.nbufs) {
        case 1: hipLaunchKernelGGL((shuffle_dense_kernel<1, false>), grid, block, lds_bytes, stream, a); break;
        case 2: hipLaunchKernelGGL((shuffle_dense_kernel<2, false>), grid, block, lds_bytes, stream, a); break;
        case 3: hipLaunchKernelGGL((shuffle_dense_kernel<3, false>), grid, block, lds_bytes, stream, a); break;
        default: hipLaunchKernelGGL((shuffle_dense_kernel<4, false>), grid, block, lds_bytes, stream, a); break;
        }
    }
    return hipGetLastError();
}

hipError_t launch_shuffle_gap(const ShuffleArgs &a, hipStream_t stream)
{
    if (a.num_tiles == 0 || a.nsegs == 0) return nothing_to_launch(a, stream);
    if (a.blocks_per_wave == 0 || a.blocks_per_wave > kWave || a.tile_coords != kGapPiece)
        return hipErrorInvalidValue;
    if ((a.blocks_per_wave & (a.blocks_per_wave - 1)) != 0) return hipErrorInvalidValue;   // lists share 512 slots evenly
    if (a.nbufs == 0 || a.nbufs > kMaxBufs) return hipErrorInvalidValue;
    const size_t per_wave = (kGapQueueCap + static_cast<size_t>(a.N) * kWave * a.nbufs) * sizeof(uint32_t);
    uint32_t waves = kWavesPerBlock;
    while (waves > 1 && per_wave * waves > 65536) waves >>= 1;
    if (per_wave * waves > 65536) return hipErrorInvalidConfiguration;
    const uint64_t nwaves = (a.num_tiles + a.blocks_per_wave - 1) / a.blocks_per_wave;
    if (a.tickets != nullptr && (a.expected != nullptr || a.nwaves != nwaves)) return hipErrorInvalidValue;
    const uint64_t blocks64 = (nwaves + waves - 1) / waves;
    if (blocks64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    const dim3 grid(static_cast<uint32_t>(blocks64)), block(kWave * waves);
    if (a.stream_stores) {
        switch (a.nbufs) {
        case 1: hipLaunchKernelGGL((shuffle_gap_kernel<1, true>), grid, block, per_wave * waves, stream, a); break;
        case 2: hipLaunchKernelGGL((shuffle_gap_kernel<2, true>), grid, block, per_wave * waves, stream, a); break;
        case 3: hipLaunchKernelGGL((shuffle_gap_kernel<3, true>), grid, block, per_wave * waves, stream, a); break;
        default: hipLaunchKernelGGL((shuffle_gap_kernel<4, true>), grid, block, per_wave * waves, stream, a); break;
        }
    } else {
        switch (a.nbufs) {
        case 1: hipLaunchKernelGGL((shuffle_gap_kernel<1, false>), grid, block, per_wave * waves, stream, a); break;
        case 2: hipLaunchKernelGGL((shuffle_gap_kernel<2, false>), grid, block, per_wave * waves, stream, a); break;
        case 3: hipLaunchKernelGGL((shuffle_gap_kernel<3, false>), grid, block, per_wave * waves, stream, a); break;
        default: hipLaunchKernelGGL((shuffle_gap_kernel<4, false>), grid, block, per_wave * waves, stream, a); break;
        }
    }
    return hipGetLastError();
}

}  // namespace wash
