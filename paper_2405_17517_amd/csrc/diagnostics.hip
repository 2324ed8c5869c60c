// Two more bandwidth-bound passes over the population, built on the same access pattern as
// the average and the EMA:
//   consensus_sqdist   out[n] = sum_g (theta[n][g] - mean[g])^2  -- the quantity of Eq. 2 and
//                      Eq. 5 and of the distance-to-consensus figures; fp64 throughout
//   weighted_average   out[g] = sum_n w[n] theta[n][g]            -- convex combinations of the
//                      models (interpolation study, soups); fp64, rounded once
#include "kernels.hpp"

#include <mutex>

namespace wash {

namespace {

constexpr int kThreads = 256;
constexpr int kWave = 64;

// Partial sums of wash_consensus_sqdist_noalloc: fixed device storage, so that the call allocates
// nothing.  Every GPU the library runs on holds its own copy, at its own address, until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[kSqdistScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
double *g_scratch_ptr[kMaxDevices] = {};     // per device: address of that device's copy of `scratch`

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

#pragma clang fp contract(off)

// Same shape as the average: a block owns V consecutive chunks of 1024 coordinates and reads the
// rows one after another (long runs per row keep DRAM pages open), fp64 products and sums in
// ascending n.
template <int V>
__global__ __launch_bounds__(kThreads) void weighted_average_kernel(const float *__restrict__ params,
                                                                    float *__restrict__ out, uint32_t N,
                                                                    uint64_t P, const Weights w)
{
    constexpr uint64_t kChunk = static_cast<uint64_t>(kThreads) * 4u;
    const uint64_t first = static_cast<uint64_t>(blockIdx.x) * kChunk * V + threadIdx.x * 4u;
    double s[V][4];
#pragma unroll
    for (int k = 0; k < V; ++k) s[k][0] = s[k][1] = s[k][2] = s[k][3] = 0.0;
    const float *row = params;
#pragma unroll 1
    for (uint32_t n = 0; n < N; ++n) {
        const double wn = w.w[n];
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const uint64_t base = first + k * kChunk;
            if (base + 4u <= P) {
                const f4u v = __builtin_nontemporal_load(reinterpret_cast<const f4u *>(row + base));
                s[k][0] += wn * static_cast<double>(v.x);
                s[k][1] += wn * static_cast<double>(v.y);
                s[k][2] += wn * static_cast<double>(v.z);
                s[k][3] += wn * static_cast<double>(v.w);
            }
        }
        row += P;
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const uint64_t base = first + k * kChunk;
        if (base + 4u <= P) {
            f4u o;
            o.x = static_cast<float>(s[k][0]);
            o.y = static_cast<float>(s[k][1]);
            o.z = static_cast<float>(s[k][2]);
            o.w = static_cast<float>(s[k][3]);
            __builtin_nontemporal_store(o, reinterpret_cast<f4u *>(out + base));
        } else if (base < P) {
            for (uint64_t g = base; g < P; ++g) {
                double t = 0.0;
                for (uint32_t n = 0; n < N; ++n) t += w.w[n] * static_cast<double>(params[static_cast<uint64_t>(n) * P + g]);
                out[g] = static_cast<float>(t);
            }
        }
    }
}

// Every block walks chunks of 1024 coordinates (grid-stride), every thread keeps N fp64
// accumulators; a fixed-shape reduction (lanes, then waves, then blocks in a second kernel)
// makes the result independent of scheduling, so two runs give the same bits.
template <int N>
__global__ __launch_bounds__(kThreads) void sqdist_partial_kernel(const float *__restrict__ params, uint64_t P,
                                                                  uint64_t g_begin, uint64_t g_end,
                                                                  double *__restrict__ partial)
{
    __shared__ double stage[kThreads / kWave][N];
    double acc[N];
#pragma unroll
    for (int n = 0; n < N; ++n) acc[n] = 0.0;
    const double den = static_cast<double>(N);
    const uint64_t span = g_end - g_begin;
    const uint64_t nchunks = (span + kThreads * 4u - 1) / (kThreads * 4u);
    for (uint64_t c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const uint64_t off = (c * kThreads + threadIdx.x) * 4u;
        if (off >= span) continue;
        const uint64_t base = g_begin + off;
        if (off + 4u <= span) {
            f4u v[N];
#pragma unroll
            for (int n = 0; n < N; ++n)
                v[n] = __builtin_nontemporal_load(reinterpret_cast<const f4u *>(params + static_cast<uint64_t>(n) * P + base));
            double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
            for (int n = 0; n < N; ++n) {
                s0 += static_cast<double>(v[n].x);
                s1 += static_cast<double>(v[n].y);
                s2 += static_cast<double>(v[n].z);
                s3 += static_cast<double>(v[n].w);
            }
            const double m0 = s0 / den, m1 = s1 / den, m2 = s2 / den, m3 = s3 / den;
#pragma unroll
            for (int n = 0; n < N; ++n) {
                const double d0 = static_cast<double>(v[n].x) - m0, d1 = static_cast<double>(v[n].y) - m1;
                const double d2 = static_cast<double>(v[n].z) - m2, d3 = static_cast<double>(v[n].w) - m3;
                acc[n] += ((d0 * d0 + d1 * d1) + d2 * d2) + d3 * d3;
            }
        } else {
            for (uint64_t g = base; g < g_end; ++g) {
                double s = 0.0;
#pragma unroll
                for (int n = 0; n < N; ++n) s += static_cast<double>(params[static_cast<uint64_t>(n) * P + g]);
                const double m = s / den;
#pragma unroll
                for (int n = 0; n < N; ++n) {
                    const double d = static_cast<double>(params[static_cast<uint64_t>(n) * P + g]) - m;
                    acc[n] += d * d;
                }
            }
        }
    }
    const uint32_t lane = threadIdx.x % kWave, wave = threadIdx.x / kWave;
#pragma unroll
    for (int n = 0; n < N; ++n) {
        double v = acc[n];
#pragma unroll
        for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_down(v, o, kWave);
        if (lane == 0) stage[wave][n] = v;
    }
    __syncthreads();
    if (threadIdx.x < N) {
        double v = stage[0][threadIdx.x];
        for (int w = 1; w < kThreads / kWave; ++w) v += stage[w][threadIdx.x];
        partial[static_cast<uint64_t>(blockIdx.x) * N + threadIdx.x] = v;
    }
}

// out[n] = sum over blocks of partial[b][n], pairwise in a fixed order (one wave per model).
__global__ __launch_bounds__(kWave) void sqdist_final_kernel(const double *__restrict__ partial, uint32_t nblocks,
                                                             uint32_t N, double *__restrict__ out)
{
    const uint32_t n = blockIdx.x;
    double v = 0.0;
    for (uint32_t b = threadIdx.x; b < nblocks; b += kWave) v += partial[static_cast<uint64_t>(b) * N + n];
#pragma unroll
    for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_down(v, o, kWave);
    if (threadIdx.x == 0) out[n] = v;
}

// Yardstick for the shuffle: independent 4-byte accesses to pseudo-random 128-byte lines of a
// large buffer, 8 per thread and round.  mode 0: loads only; 1: stores only; 2: load, then store a
// value to the same place (the access pattern of a sparse shuffle without any of its arithmetic);
// 3: stores of whole 64-byte pieces (four neighbouring threads write 16 bytes each to one
// pseudo-random half line): the memory side takes these without filling the piece first.
__device__ __forceinline__ uint32_t probe_mix(uint32_t x)
{
    x ^= x >> 16;
    x *= 0x7FEB352Du;
    x ^= x >> 15;
    x *= 0x846CA68Bu;
    x ^= x >> 16;
    return x;
}

typedef uint32_t u4a __attribute__((ext_vector_type(4)));

template <int MODE>
__global__ __launch_bounds__(kThreads) void scatter_probe_kernel(uint32_t *__restrict__ buf, uint32_t line_mask,
                                                                 uint32_t rounds, uint32_t *__restrict__ sink)
{
    constexpr int K = 8;
    const uint32_t tid = blockIdx.x * kThreads + threadIdx.x;
    uint32_t acc = tid;
    if (MODE == 3) {
        const uint32_t group = tid >> 2, part = tid & 3u;
        for (uint32_t r = 0; r < rounds; ++r) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const uint32_t h = probe_mix(group * 2654435761u + r * 40503u + k * 0x9E3779B9u);
                const uint32_t line = h & line_mask;
                const uint32_t half = probe_mix(h) & 1u;
                u4a *p = reinterpret_cast<u4a *>(buf + static_cast<uint64_t>(line) * 32u + half * 16u) + part;
                const u4a v = {h, h + 1u, h + 2u, h + 3u};
                *p = v;
            }
        }
        return;
    }
    for (uint32_t r = 0; r < rounds; ++r) {
        uint32_t *p[K];
        uint32_t v[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const uint32_t line = probe_mix(tid * 2654435761u + r * 40503u + k * 0x9E3779B9u) & line_mask;
            p[k] = buf + static_cast<uint64_t>(line) * 32u + (probe_mix(line) & 31u);   // inside line `line`
        }
        if (MODE != 1) {
#pragma unroll
            for (int k = 0; k < K; ++k) v[k] = __builtin_nontemporal_load(p[k]);
#pragma unroll
            for (int k = 0; k < K; ++k) acc ^= v[k];
        }
        if (MODE != 0) {
#pragma unroll
            for (int k = 0; k < K; ++k) *p[k] = (MODE == 2) ? v[(k + 1) % K] : acc + k;
        }
    }
    if (acc == 0x12345678u) sink[0] = acc;   // keeps the loads alive
}

template <int N>
hipError_t run_sqdist(const float *params, uint64_t P, uint64_t g_begin, uint64_t g_end, double *partial,
                      uint32_t nblocks, double *out, hipStream_t stream)
{
    hipLaunchKernelGGL(sqdist_partial_kernel<N>, dim3(nblocks), dim3(kThreads), 0, stream, params, P, g_begin, g_end,
                       partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sqdist_final_kernel, dim3(N), dim3(kWave), 0, stream, partial, nblocks, static_cast<uint32_t>(N), out);
    return hipGetLastError();
}

}  // namespace

// Address of the CURRENT device's copy of the static scratch array (looked up once per device).
hipError_t static_sqdist_scratch(int device, double **out)
{
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[device] == nullptr) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

uint32_t sqdist_blocks(uint64_t span)
{
    const uint64_t nchunks = (span + kThreads * 4u - 1) / (kThreads * 4u);
    return static_cast<uint32_t>(nchunks < kSqdistMaxBlocks ? (nchunks ? nchunks : 1) : kSqdistMaxBlocks);
}

hipError_t launch_scatter_probe(uint32_t *buf, uint64_t lines, int mode, uint32_t rounds, uint32_t blocks,
                                uint32_t *sink, hipStream_t stream)
{
    if (lines == 0 || (lines & (lines - 1)) != 0 || lines > (1ull << 32) || blocks == 0 || blocks > (1u << 20))
        return hipErrorInvalidValue;
    const uint32_t mask = static_cast<uint32_t>(lines - 1);
    switch (mode) {
    case 0: hipLaunchKernelGGL(scatter_probe_kernel<0>, dim3(blocks), dim3(kThreads), 0, stream, buf, mask, rounds, sink); break;
    case 1: hipLaunchKernelGGL(scatter_probe_kernel<1>, dim3(blocks), dim3(kThreads), 0, stream, buf, mask, rounds, sink); break;
    case 2: hipLaunchKernelGGL(scatter_probe_kernel<2>, dim3(blocks), dim3(kThreads), 0, stream, buf, mask, rounds, sink); break;
    case 3: hipLaunchKernelGGL(scatter_probe_kernel<3>, dim3(blocks), dim3(kThreads), 0, stream, buf, mask, rounds, sink); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_weighted_average(const float *params, float *out, uint32_t N, uint64_t P, const Weights &w,
                                   hipStream_t stream)
{
    const int V = average_chunks_for(N, P) >= 4 ? 8 : 1;
    const uint64_t per_block = static_cast<uint64_t>(kThreads) * 4u * V;
    const uint64_t blocks = (P + per_block - 1) / per_block;
    if (N == 0 || N > 32 || blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    if (V == 8)
        hipLaunchKernelGGL(weighted_average_kernel<8>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, stream,
                           params, out, N, P, w);
    else
        hipLaunchKernelGGL(weighted_average_kernel<1>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, stream,
                           params, out, N, P, w);
    return hipGetLastError();
}

#define WASH_FOR_EACH_N(X)                                                                         \
    X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17)   \
    X(18) X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)

hipError_t launch_sqdist(const float *params, uint32_t N, uint64_t P, uint64_t g_begin, uint64_t g_end,
                         double *partial, double *out, hipStream_t stream)
{
    const uint32_t nblocks = sqdist_blocks(g_end - g_begin);
    switch (N) {
#define X(n) case n: return run_sqdist<n>(params, P, g_begin, g_end, partial, nblocks, out, stream);
        WASH_FOR_EACH_N(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

}  // namespace wash
