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
#include "kernels.hpp"

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

template <int N, bool NT>
__global__ __launch_bounds__(kThreads) void ema_kernel(float *__restrict__ params, uint64_t P, double alpha)
{
    const uint64_t base = (static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x) * 4u;
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

inline bool grid_for(uint64_t P, dim3 &grid)
{
    const uint64_t threads = (P + 3u) / 4u;
    const uint64_t blocks = (threads + kThreads - 1) / kThreads;
    if (blocks == 0 || blocks > 0x7FFFFFFFull) return false;
    grid = dim3(static_cast<uint32_t>(blocks));
    return true;
}

template <int N>
hipError_t run_ema(float *params, uint64_t P, double alpha, bool nt, hipStream_t stream)
{
    dim3 grid;
    if (!grid_for(P, grid)) return hipErrorInvalidConfiguration;
    if (nt) hipLaunchKernelGGL((ema_kernel<N, true>), grid, dim3(kThreads), 0, stream, params, P, alpha);
    else hipLaunchKernelGGL((ema_kernel<N, false>), grid, dim3(kThreads), 0, stream, params, P, alpha);
    return hipGetLastError();
}

}  // namespace

#define WASH_FOR_EACH_N(X)                                                                         \
    X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13) X(14) X(15) X(16) X(17)   \
    X(18) X(19) X(20) X(21) X(22) X(23) X(24) X(25) X(26) X(27) X(28) X(29) X(30) X(31) X(32)

hipError_t launch_copy(const float *src, float *dst, uint64_t n, hipStream_t stream)
{
    dim3 grid;
    if (!grid_for(n, grid)) return hipErrorInvalidConfiguration;
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

hipError_t launch_average(const float *params, float *out, uint32_t N, uint64_t P, int chunks, hipStream_t stream)
{
    if (N == 0) return hipErrorInvalidValue;
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
