// wash_shuffle kernel for gfx950: the shuffling step of WASH (Sec. 3, Eq. 3;
// Alg. 1, shuffling step), with the optimizer state moved along (WASH+Opt).
//
// One wavefront owns one tile of consecutive coordinates and works alone (no
// workgroup barrier anywhere):
//   scan     each lane draws the mask words of 4 consecutive coordinates with
//            one Philox call and compares them with the segment threshold;
//            the Bernoulli mask is never written to memory.
//   compact  selected coordinates are appended to a small per-wave LDS queue
//            through ballot + lane-prefix counts, so the expensive part below
//            runs on dense lanes and HBM traffic follows p*N*P, not N*P.
//   permute  whenever 64 coordinates are queued (and once at the end) each
//            lane takes one coordinate: its N values (and N momentum values)
//            are gathered into an LDS slab [N][64], the descending
//            Fisher-Yates walk swaps slab rows in place, and because slot i is
//            final after step i its value is stored to row i right there.
// Everything random is integer arithmetic, so the result is bit-identical to
// any other implementation of the same stream.
#include "kernels.hpp"
#include "philox.hpp"

namespace wash {

namespace {

constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
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

// Gather, permute and scatter up to 64 queued coordinates, one per lane.
template <bool kMomentum>
__device__ __forceinline__ void permute_batch(const ShuffleArgs &a, uint64_t tile_begin,
                                              const uint32_t *queue, uint32_t nbatch,
                                              uint32_t *slab, uint32_t *slab_m)
{
    const uint32_t lane = lane_id();
    if (lane >= nbatch) return;
    const uint64_t g = tile_begin + queue[lane];
    const uint32_t N = a.N;
    const uint64_t P = a.P;
    uint32_t *col = a.params + g;
    uint32_t *col_m = kMomentum ? a.momentum + g : nullptr;

    // gather the column(s) into the slab: slab[n][lane]
#pragma unroll 8
    for (uint32_t n = 0; n < N; ++n) {
        slab[n * kWave + lane] = col[static_cast<uint64_t>(n) * P];
        if (kMomentum) slab_m[n * kWave + lane] = col_m[static_cast<uint64_t>(n) * P];
    }

    // descending Fisher-Yates on the values themselves: swapping slab rows i and j keeps
    // slab[n] == old[perm[n]]; row i is final after step i and goes straight to memory
    const uint32_t g_lo = static_cast<uint32_t>(g), g_hi = static_cast<uint32_t>(g >> 32);
    uint32_t i = N - 1;
    for (uint32_t call = 0; i > 0; ++call) {
        const Words4 r = philox4x32_10(g_lo, g_hi, a.step, 1u + call, a.key_lo, a.key_hi);
        const uint32_t w[4] = {r.w0, r.w1, r.w2, r.w3};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (i == 0) break;
            const uint32_t j = __umulhi(w[k], i + 1u);
            const uint32_t vi = slab[i * kWave + lane];
            const uint32_t vj = slab[j * kWave + lane];
            col[static_cast<uint64_t>(i) * P] = vj;
            slab[j * kWave + lane] = vi;
            if (kMomentum) {
                const uint32_t mi = slab_m[i * kWave + lane];
                const uint32_t mj = slab_m[j * kWave + lane];
                col_m[static_cast<uint64_t>(i) * P] = mj;
                slab_m[j * kWave + lane] = mi;
            }
            --i;
        }
    }
    col[0] = slab[lane];
    if (kMomentum) col_m[0] = slab_m[lane];
}

template <bool kMomentum>
__global__ __launch_bounds__(kWave * kWavesPerBlock) void shuffle_kernel(const ShuffleArgs a)
{
    extern __shared__ uint32_t lds[];
    const uint32_t lane = lane_id();
    const uint32_t wave_in_block = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const uint64_t tile = static_cast<uint64_t>(blockIdx.x) * kWavesPerBlock + wave_in_block;
    if (tile >= a.num_tiles) return;
    const uint32_t first = a.tile_first[tile];
    if (first == kNoSegment) return;

    const uint32_t slab_words = a.N * kWave;
    const uint32_t per_wave = kQueueCap + slab_words * (kMomentum ? 2u : 1u);
    uint32_t *queue = lds + wave_in_block * per_wave;
    uint32_t *slab = queue + kQueueCap;
    uint32_t *slab_m = slab + slab_words;

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
        const Words4 r = philox4x32_10(static_cast<uint32_t>(quad), static_cast<uint32_t>(quad >> 32),
                                       a.step, 0u, a.key_lo, a.key_hi);
        const uint32_t w[4] = {r.w0, r.w1, r.w2, r.w3};
        bool sel[4];
        if (uniform) {
#pragma unroll
            for (int k = 0; k < 4; ++k) sel[k] = (w[k] <= seg0.thr_m1) && (g0 + k < tile_end);
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint64_t g = g0 + k;
                // coordinates of a lane only grow, so the cursor only moves forward
                while (walk < a.nsegs && a.segs[walk].end <= g) ++walk;
                bool s = false;
                if (walk < a.nsegs && g < tile_end) {
                    const DevSegment sg = a.segs[walk];
                    s = (sg.begin <= g) && (w[k] <= sg.thr_m1);
                }
                sel[k] = s;
            }
        }
        if (__ballot(sel[0] | sel[1] | sel[2] | sel[3]) == 0) continue;

#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const uint64_t m = __ballot(sel[k]);
            if (sel[k]) queue[queued + lanes_below(m)] = static_cast<uint32_t>(g0 + k - tile_begin);
            queued += __popcll(m);
        }
        while (queued >= kWave) {
            wave_lds_sync();
            permute_batch<kMomentum>(a, tile_begin, queue + (queued - kWave), kWave, slab, slab_m);
            queued -= kWave;
            selected += kWave;
            wave_lds_sync();
        }
    }
    if (queued > 0) {
        wave_lds_sync();
        permute_batch<kMomentum>(a, tile_begin, queue, queued, slab, slab_m);
        selected += queued;
    }
    if (a.selected_count != nullptr && selected != 0 && lane == 0)
        atomicAdd(a.selected_count, static_cast<unsigned long long>(selected));
}

}  // namespace

hipError_t launch_shuffle(const ShuffleArgs &a, hipStream_t stream)
{
    if (a.num_tiles == 0 || a.nsegs == 0) return hipSuccess;
    const uint64_t blocks64 = (a.num_tiles + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks64 > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    const dim3 grid(static_cast<uint32_t>(blocks64)), block(kWave * kWavesPerBlock);
    const size_t per_wave = kQueueCap + static_cast<size_t>(a.N) * kWave * (a.momentum ? 2 : 1);
    const size_t lds_bytes = per_wave * kWavesPerBlock * sizeof(uint32_t);
    if (a.momentum)
        hipLaunchKernelGGL(shuffle_kernel<true>, grid, block, lds_bytes, stream, a);
    else
        hipLaunchKernelGGL(shuffle_kernel<false>, grid, block, lds_bytes, stream, a);
    return hipGetLastError();
}

}  // namespace wash
