// wash_average (Alg. 1 output line) and papa_ema (Sec. 3, Eq. 1) for gfx950.
//
// Both are pure streaming passes bound by HBM bandwidth: every thread owns 4
// consecutive coordinates, reads 16 bytes per row, accumulates in fp64 in
// ascending n (the same order and precision as the plain definition, so the
// fp32 result is the correctly rounded one) and writes 16 bytes per row.  For
// the EMA N is a template parameter so the N values stay in registers: it reads
// and writes each element exactly once.  Rows are P elements apart and P need not be a multiple
// of 4, so the 16-byte accesses are only 4-byte aligned; gfx950 global memory
// accepts that.
//
// Launch shape in the streaming regime (population beyond the 256 MB Infinity Cache).  What these
// kernels are up against is not latency but DRAM page locality: all blocks in flight read (and write)
// a window of every row at once, and the wider that window, the more DRAM pages are open at a time
// and the more often a page is closed before its neighbours' requests arrive.  Measured on MI355X,
// N = 8, P = 1.1e9: the EMA reaches 68 % of 8 TB/s at full occupancy (32 wavefronts per compute
// unit), 74 % at 8-12, 79 % at 5, 55 % at 2-3; the best point sits where about 40 KB (EMA) to 60 KB
// (average) of loads are in flight per compute unit, whatever N is.  Occupancy is therefore capped on
// purpose, by asking for dynamic LDS the kernel never touches (160 KB per compute unit: a block that
// asks for 160/k KB leaves room for k blocks).  The hardware dispatcher hands out blocks in order
// as others retire, which keeps the window compact; persistent grid-stride variants let it spread
// (fast wavefronts run ahead) and measured 55-65 %.
// Rows whose byte pitch is not a multiple of 128 cost 6-10 points: the first and last cache line of
// every per-row piece is then shared with another block, read twice and written in two partial
// pieces.  Blocks of 256 threads (4 KB per row) have a quarter of the seams of single wavefronts
// (1 KB per row), so they are used there; aligned rows do best with single-wavefront blocks.
#include "kernels.hpp"

#include <atomic>

namespace wash {

namespace {

constexpr int kThreads = 256;

typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));

// Non-temporal accesses stream past the caches.  The average always uses them (it never
// re-reads anything).  The in-place EMA uses them once the population exceeds the 256 MB
// Infinity Cache; below that, plain accesses let its stores hit the lines its loads brought in.
template <bool NT>
__device__ __forceinline__ f4u load4(const float *p)
{
    if (NT) return __builtin_nontemporal_load(reinterpret_cast<const f4u *>(p));
    return *reinterpret_cast<const f4u *>(p);
}
template <bool NT>
__device__ __forceinline__ void store4(float *p, f4u v)
{
    if (NT) __builtin_nontemporal_store(v, reinterpret_cast<f4u *>(p));
    else *reinterpret_cast<f4u *>(p) = v;
}

// fp64 arithmetic is kept unfused so that it matches the definition operation by operation
#pragma clang fp contract(off)

// A block owns V consecutive chunks of 1024 coordinates and reads the rows strictly one after
// another: V 16-byte loads in flight per thread (the 32 KB vector L1 bounds a compute unit to 256
// lines in flight anyway), V*4 fp64 accumulators, one burst of V*4 KB of output at the end.
// Long runs per row and per block keep DRAM pages open: with V = 8 the N = 20 average measured
// 80 % of peak against 73 % with V = 1 -- its 5 % of writes, sprinkled among 20 read streams,
// otherwise cost 17 % of the time (the same kernel without its store reads at 83 %).  V = 8 needs
// many rows and enough blocks to fill the chip several times over; otherwise V = 1 is faster.
// N is a run-time value.
template <int V>
__global__ __launch_bounds__(kThreads) void average_kernel(const float *__restrict__ params,
                                                           float *__restrict__ out, uint32_t N, uint64_t P)
{
    constexpr uint64_t kChunk = static_cast<uint64_t>(kThreads) * 4u;
    const uint64_t first = static_cast<uint64_t>(blockIdx.x) * kChunk * V + threadIdx.x * 4u;
    const double den = static_cast<double>(N);
    double s[V][4];
#pragma unroll
    for (int k = 0; k < V; ++k) s[k][0] = s[k][1] = s[k][2] = s[k][3] = 0.0;
    const float *row = params;
#pragma unroll 1
    for (uint32_t n = 0; n < N; ++n) {
#pragma unroll
        for (int k = 0; k < V; ++k) {
            const uint64_t base = first + k * kChunk;
            if (base + 4u <= P) {
                const f4u v = load4<true>(row + base);
                s[k][0] += static_cast<double>(v.x);
                s[k][1] += static_cast<double>(v.y);
                s[k][2] += static_cast<double>(v.z);
                s[k][3] += static_cast<double>(v.w);
            }
        }
        row += P;
    }
#pragma unroll
    for (int k = 0; k < V; ++k) {
        const uint64_t base = first + k * kChunk;
        if (base + 4u <= P) {
            f4u o;
            o.x = static_cast<float>(s[k][0] / den);
            o.y = static_cast<float>(s[k][1] / den);
            o.z = static_cast<float>(s[k][2] / den);
            o.w = static_cast<float>(s[k][3] / den);
            store4<true>(out + base, o);
        } else if (base < P) {
            // the last, ragged float4 of a row
            for (uint64_t g = base; g < P; ++g) {
                double t = 0.0;
                for (uint32_t n = 0; n < N; ++n) t += static_cast<double>(params[static_cast<uint64_t>(n) * P + g]);
                out[g] = static_cast<float>(t / den);
            }
        }
    }
}

// The average with all N loads of a thread in flight at once (N a template parameter), for the
// streaming regime with N >= 5: same sums in the same order, launched with capped occupancy.
template <int N, int BLOCK>
__global__ __launch_bounds__(BLOCK) void average_inflight_kernel(const float *__restrict__ params,
                                                                 float *__restrict__ out, uint64_t P)
{
    const uint64_t base = (static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 4u;
    if (base >= P) return;
    const double den = static_cast<double>(N);
    if (base + 4u <= P) {
        f4u v[N];
#pragma unroll
        for (int n = 0; n < N; ++n) v[n] = load4<true>(params + static_cast<uint64_t>(n) * P + base);
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (int n = 0; n < N; ++n) {
            s0 += static_cast<double>(v[n].x);
            s1 += static_cast<double>(v[n].y);
            s2 += static_cast<double>(v[n].z);
            s3 += static_cast<double>(v[n].w);
        }
        f4u o;
        o.x = static_cast<float>(s0 / den);
        o.y = static_cast<float>(s1 / den);
        o.z = static_cast<float>(s2 / den);
        o.w = static_cast<float>(s3 / den);
        store4<true>(out + base, o);
    } else {
        for (uint64_t g = base; g < P; ++g) {
            double t = 0.0;
#pragma unroll
            for (int n = 0; n < N; ++n) t += static_cast<double>(params[static_cast<uint64_t>(n) * P + g]);
            out[g] = static_cast<float>(t / den);
        }
    }
}

template <int N, bool NT, int BLOCK>
__global__ __launch_bounds__(BLOCK) void ema_kernel(float *__restrict__ params, uint64_t P, double alpha)
{
    const uint64_t base = (static_cast<uint64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 4u;
    if (base >= P) return;
    const double den = static_cast<double>(N);
    const double beta = 1.0 - alpha;
    if (base + 4u <= P) {
        f4u v[N];
#pragma unroll
        for (int n = 0; n < N; ++n)
            v[n] = load4<NT>(params + static_cast<uint64_t>(n) * P + base);
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
#pragma unroll
        for (int n = 0; n < N; ++n) {
            s0 += static_cast<double>(v[n].x);
            s1 += static_cast<double>(v[n].y);
            s2 += static_cast<double>(v[n].z);
            s3 += static_cast<double>(v[n].w);
        }
        const double m0 = beta * (s0 / den), m1 = beta * (s1 / den), m2 = beta * (s2 / den), m3 = beta * (s3 / den);
#pragma unroll
        for (int n = 0; n < N; ++n) {
            f4u o;
            o.x = static_cast<float>(alpha * static_cast<double>(v[n].x) + m0);
            o.y = static_cast<float>(alpha * static_cast<double>(v[n].y) + m1);
            o.z = static_cast<float>(alpha * static_cast<double>(v[n].z) + m2);
            o.w = static_cast<float>(alpha * static_cast<double>(v[n].w) + m3);
            store4<NT>(params + static_cast<uint64_t>(n) * P + base, o);
        }
    } else {
        for (uint64_t g = base; g < P; ++g) {
            double s = 0.0;
#pragma unroll
            for (int n = 0; n < N; ++n) s += static_cast<double>(params[static_cast<uint64_t>(n) * P + g]);
            const double m = beta * (s / den);
#pragma unroll
            for (int n = 0; n < N; ++n) {
                float *q = params + static_cast<uint64_t>(n) * P + g;
                *q = static_cast<float>(alpha * static_cast<double>(*q) + m);
            }
        }
    }
}

// Plain streaming copy: the yardstick for what a one-pass kernel can reach on this chip.
__global__ __launch_bounds__(kThreads) void copy_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                        uint64_t n)
{
    const uint64_t base = (static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4u;
    if (base >= n) return;
    if (base + 4u <= n) {
        const f4u v = __builtin_nontemporal_load(reinterpret_cast<const f4u *>(src + base));
        __builtin_nontemporal_store(v, reinterpret_cast<f4u *>(dst + base));
    } else {
        for (uint64_t g = base; g < n; ++g) dst[g] = src[g];
    }
}

inline bool grid_for(uint64_t P, int block, dim3 &grid)
{
    const uint64_t threads = (P + 3u) / 4u;
    const uint64_t blocks = (threads + block - 1) / block;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return false;
    grid = dim3(static_cast<uint32_t>(blocks));
    return true;
}

// Dynamic LDS (never touched by the kernel) that lets exactly `blocks_per_cu` blocks share the 160 KB of a
// compute unit; 0 = no cap.  Valid for 1 .. 20 blocks.
constexpr uint32_t kLdsPerCu = 160u * 1024u;
inline uint32_t occupancy_pad_bytes(int blocks_per_cu)
{
    if (blocks_per_cu <= 0 || blocks_per_cu > 20) return 0;
    return (kLdsPerCu - 1024u) / static_cast<uint32_t>(blocks_per_cu) / 256u * 256u;
}

// More than 64 KB of dynamic LDS has to be allowed per kernel (once per device).
constexpr int kMaxDevices = 64;
template <auto Kernel>
hipError_t allow_large_lds()
{
    static std::atomic<bool> done[kMaxDevices];
    int device = 0;
    hipError_t e = hipGetDevice(&device);
    if (e != hipSuccess) return e;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[device].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(kLdsPerCu - 1024u));
    if (e == hipSuccess) done[device].store(true, std::memory_order_release);
    return e;
}

struct LaunchShape {
    int block;           // threads per block: 64 or 256
    int blocks_per_cu;   // occupancy cap, 0 = none
};

// Measured best shapes (MI355X; see the note at the top of this file).  `aligned`: the byte pitch of a row is a
// multiple of 128.
inline LaunchShape ema_shape(uint32_t N, bool aligned)
{
    const int waves = static_cast<int>((40u + N / 2u) / N);            // about 40 KB of loads in flight per compute unit
    if (aligned || N <= 4) return LaunchShape{64, waves < 5 ? 5 : (waves > 17 ? 17 : waves)};
    const int blocks = static_cast<int>((10u + N / 2u) / N);           // the same in blocks of four wavefronts
    return LaunchShape{256, blocks < 1 ? 1 : blocks};
}
inline LaunchShape average_shape(uint32_t N, bool aligned)
{
    if (aligned) {
        const int waves = static_cast<int>((60u + N / 2u) / N);        // about 60 KB in flight
        return LaunchShape{64, waves < 5 ? 5 : (waves > 16 ? 16 : waves)};
    }
    const int blocks = static_cast<int>((16u + N / 2u) / N);
    return LaunchShape{256, blocks < 1 ? 1 : (blocks > 4 ? 4 : blocks)};
}

template <int N>
hipError_t run_ema(float *params, uint64_t P, double alpha, bool nt, hipStream_t stream)
{
    dim3 grid;
    if (!nt) {
        // population inside the Infinity Cache: plain accesses, full occupancy
        if (!grid_for(P, kThreads, grid)) return hipErrorInvalidConfiguration;
        hipLaunchKernelGGL((ema_kernel<N, false, kThreads>), grid, dim3(kThreads), 0, stream, params, P, alpha);
        return hipGetLastError();
    }
    const LaunchShape shape = ema_shape(N, (P % 32u) == 0);
    const uint32_t pad = occupancy_pad_bytes(shape.blocks_per_cu);
    if (!grid_for(P, shape.block, grid)) return hipErrorInvalidConfiguration;
    if (shape.block == 64) {
        if (pad > 65536u)
            if (const hipError_t e = allow_large_lds<ema_kernel<N, true, 64>>()) return e;
        hipLaunchKernelGGL((ema_kernel<N, true, 64>), grid, dim3(64), pad, stream, params, P, alpha);
    } else {
        if (pad > 65536u)
            if (const hipError_t e = allow_large_lds<ema_kernel<N, true, kThreads>>()) return e;
        hipLaunchKernelGGL((ema_kernel<N, true, kThreads>), grid, dim3(kThreads), pad, stream, params, P, alpha);
    }
    return hipGetLastError();
}

template <int N>
hipError_t run_average_inflight(const float *params, float *out, uint64_t P, hipStream_t stream)
{
    const LaunchShape shape = average_shape(N, (P % 32u) == 0);
    const uint32_t pad = occupancy_pad_bytes(shape.blocks_per_cu);
    dim3 grid;
    if (!grid_for(P, shape.block, grid)) return hipErrorInvalidConfiguration;
    if (shape.block == 64) {
        if (pad > 65536u)
            if (const hipError_t e = allow_large_lds<average_inflight_kernel<N, 64>>()) return e;
        hipLaunchKernelGGL((average_inflight_kernel<N, 64>), grid, dim3(64), pad, stream, params, out, P);
    } else {
        if (pad > 65536u)
            if (const hipError_t e = allow_large_lds<average_inflight_kernel<N, kThreads>>()) return e;
        hipLaunchKernelGGL((average_inflight_kernel<N, kThreads>), grid, dim3(kThreads), pad, stream, params, out, P);
    }
    return hipGetLastError();
}

}  // namespace

#define WASH_FOR_EACH_N(X)                                                                         \
    X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17)   \
    X(18) X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)

hipError_t launch_copy(const float *src, float *dst, uint64_t n, hipStream_t stream)
{
    dim3 grid;
    if (!grid_for(n, kThreads, grid)) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(copy_kernel, grid, dim3(kThreads), 0, stream, src, dst, n);
    return hipGetLastError();
}

template <int V>
hipError_t run_average(const float *params, float *out, uint32_t N, uint64_t P, hipStream_t stream)
{
    const uint64_t per_block = static_cast<uint64_t>(kThreads) * 4u * V;
    const uint64_t blocks = (P + per_block - 1) / per_block;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(average_kernel<V>, dim3(static_cast<uint32_t>(blocks)), dim3(kThreads), 0, stream, params, out, N, P);
    return hipGetLastError();
}

hipError_t launch_average(const float *params, float *out, uint32_t N, uint64_t P, int chunks, bool streaming,
                          hipStream_t stream)
{
    if (N == 0) return hipErrorInvalidValue;
    if (chunks == 0) {
        // automatic: beyond the Infinity Cache and from five models on, all N loads in flight under an occupancy cap;
        // otherwise the rows one after the other at full occupancy
        if (N >= 5 && streaming) {
            switch (N) {
#define X(n) case n: return run_average_inflight<n>(params, out, P, stream);
                WASH_FOR_EACH_N(X)
#undef X
            default: return hipErrorInvalidValue;
            }
        }
        return run_average<1>(params, out, N, P, stream);
    }
    switch (chunks) {
    case 8: return run_average<8>(params, out, N, P, stream);
    case 4: return run_average<4>(params, out, N, P, stream);
    case 2: return run_average<2>(params, out, N, P, stream);
    default: return run_average<1>(params, out, N, P, stream);
    }
}

hipError_t launch_ema(float *params, uint32_t N, uint64_t P, float alpha, bool nt, hipStream_t stream)
{
    switch (N) {
#define X(n) case n: return run_ema<n>(params, P, static_cast<double>(alpha), nt, stream);
        WASH_FOR_EACH_N(X)
#undef X
    default: return hipErrorInvalidValue;
    }
}

}  // namespace wash
