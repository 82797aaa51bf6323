// Resident series store (Sec. 4.1 of the paper, GPU-Index-Batching: the data is migrated to GPU
// memory once; Eq. 2: a single copy of the data is kept).  Device-side helpers used while the
// series is loaded: the optional fp32 -> bf16 storage rounding and the per-feature mean /
// population standard deviation (Algorithm 1 standardises with the mean and standard deviation;
// its caption allows other ranges than its own, here every feature over the whole series).
#include "pgti_internal.h"

namespace pgti {
namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Round to nearest, ties to even, on the upper 16 bits.  NaN keeps sign and upper payload and
// gets the quiet bit so that it cannot round to infinity.
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

__global__ void __launch_bounds__(kThreads) store_bf16_kernel(const float* __restrict__ src,
                                                              uint16_t* __restrict__ dst, size_t count) {
    const size_t quads = count / 4;
    const size_t stride = static_cast<size_t>(gridDim.x) * kThreads;
    for (size_t q = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x; q < quads; q += stride) {
        f32x4 v = reinterpret_cast<const f32x4*>(src)[q];
        u32x2 o;
        o.x = bf16_bits(v.x) | (bf16_bits(v.y) << 16);
        o.y = bf16_bits(v.z) | (bf16_bits(v.w) << 16);
        reinterpret_cast<u32x2*>(dst)[q] = o;
    }
    // tail of count % 4 elements
    const size_t tail0 = quads * 4;
    if (blockIdx.x == 0 && threadIdx.x < count - tail0)
        dst[tail0 + threadIdx.x] = static_cast<uint16_t>(bf16_bits(src[tail0 + threadIdx.x]));
}

// Time of day of absolute timestep t: (t mod period) / period, the quotient taken in binary32.
__device__ __forceinline__ float time_of_day(int64_t t, int32_t period) {
    return static_cast<float>(static_cast<int32_t>(t % period)) / static_cast<float>(period);
}

// Writes rows of the resident series from a source chunk with fewer features: out[t, node, f] =
// src[t, node, f] for f < F_src, and the time-of-day value of the row for f == F_src (stage 1 of the
// preprocessing: the same value for every node of a timestep).  One output element per thread.
template <bool OUT_BF16>
__global__ void __launch_bounds__(kThreads) assemble_rows_kernel(const float* __restrict__ src, int64_t rows,
                                                                 int32_t N, int32_t F_src, int32_t F, int64_t row0,
                                                                 int32_t period, void* __restrict__ dst) {
    const int64_t total = rows * N * F;
    const int64_t stride = static_cast<int64_t>(gridDim.x) * kThreads;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x; i < total; i += stride) {
        const int64_t cell = i / F;  // (row, node)
        const int32_t f = static_cast<int32_t>(i - cell * F);
        const float v = (f < F_src) ? src[cell * F_src + f] : time_of_day(row0 + cell / N, period);
        if constexpr (OUT_BF16) static_cast<uint16_t*>(dst)[i] = static_cast<uint16_t>(bf16_bits(v));
        else static_cast<float*>(dst)[i] = v;
    }
}

// One wave per (row, feature): lane l adds the nodes l, l+64, ... in node order, then the 64 lane
// sums are combined in a fixed butterfly.  The order depends on nothing but N, so the result does
// not depend on how the series was cut into chunks.  The chunk holds F_src features per node; a
// feature f >= F_src is the synthesised time-of-day channel.
__global__ void __launch_bounds__(kThreads) row_sums_kernel(const float* __restrict__ chunk, int64_t rows,
                                                            int32_t N, int32_t F, int32_t F_src, int32_t period,
                                                            int64_t row0, const double* __restrict__ mean64,
                                                            double* __restrict__ row_acc) {
    const uint32_t lane = threadIdx.x & 63u;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
    if (wave >= rows * F) return;  // whole waves leave together
    const int64_t row = wave / F;
    const int32_t f = static_cast<int32_t>(wave % F);
    const bool synth = f >= F_src;
    const float* p = chunk + row * static_cast<int64_t>(N) * F_src + (synth ? 0 : f);
    const double tod = synth ? static_cast<double>(time_of_day(row0 + row, period)) : 0.0;
    const double mu = mean64 ? mean64[f] : 0.0;
    double acc = 0.0;
    auto add = [&](double v) {
        if (mean64) {
            const double d = v - mu;
            acc += d * d;
        } else {
            acc += v;
        }
    };
    if (synth) {
        // same value for every node of the row; same additions, in the same order, as for a stored feature
        for (int32_t node = lane; node < N; node += 64) add(tod);
    } else {
        // Sixteen loads are issued before the first is added (a wave has a whole row to itself, so
        // its load latencies would otherwise run one after the other); the additions keep the node
        // order.  The loads are unconditional inside this branch so that they can be in flight together.
        constexpr int32_t kAhead = 16;
        int32_t node = lane;
        for (; node + 64 * (kAhead - 1) < N; node += 64 * kAhead) {
            float v[kAhead];
#pragma unroll
            for (int32_t u = 0; u < kAhead; ++u) v[u] = p[static_cast<int64_t>(node + 64 * u) * F_src];
#pragma unroll
            for (int32_t u = 0; u < kAhead; ++u) add(static_cast<double>(v[u]));
        }
        for (; node < N; node += 64) add(static_cast<double>(p[static_cast<int64_t>(node) * F_src]));
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) row_acc[(row0 + row) * F + f] = acc;
}

// Algorithm 1's statistics: one scalar over every element of x_train, the first n_train windows of
// the stacked x.  Row t belongs to w_t = min(t, n_train-1) - max(0, t-P+1) + 1 of those windows, so
// the sum over x_train is the w_t-weighted sum of the row sums, features mixed.  One workgroup;
// thread i takes rows i, i+256, ... in time order, then a fixed LDS tree.  The scalar is written
// to all F entries.
__global__ void __launch_bounds__(kThreads) reduce_rows_alg1_kernel(const double* __restrict__ row_acc, int32_t F,
                                                                    int64_t n_train, int32_t P, double count,
                                                                    int take_sqrt, double* __restrict__ out64,
                                                                    float* __restrict__ out32) {
    __shared__ double part[kThreads];
    const int64_t last_row = n_train + P - 1;  // rows [0, last_row) appear in x_train
    double acc = 0.0;
    auto row_total = [&](int64_t t) {
        double total = 0.0;
        for (int32_t f = 0; f < F; ++f) total += row_acc[t * F + f];
        return total;
    };
    auto add_row = [&](int64_t t, double total) {
        const int64_t hi = t < n_train - 1 ? t : n_train - 1;
        const int64_t lo = t - P + 1 > 0 ? t - P + 1 : 0;
        acc += static_cast<double>(hi - lo + 1) * total;
    };
    // rows are read eight ahead (one workgroup walks the whole table); the additions keep the row order
    constexpr int kAhead = 8;
    int64_t t = threadIdx.x;
    for (; t + static_cast<int64_t>(kThreads) * (kAhead - 1) < last_row; t += static_cast<int64_t>(kThreads) * kAhead) {
        double v[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) v[u] = 0.0;
        for (int32_t f = 0; f < F; ++f) {  // features in order for every row, eight rows' loads in flight
#pragma unroll
            for (int u = 0; u < kAhead; ++u) v[u] += row_acc[(t + static_cast<int64_t>(kThreads) * u) * F + f];
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u) add_row(t + static_cast<int64_t>(kThreads) * u, v[u]);
    }
    for (; t < last_row; t += kThreads) add_row(t, row_total(t));
    part[threadIdx.x] = acc;
    __syncthreads();
    for (uint32_t off = kThreads / 2; off >= 1; off >>= 1) {
        if (threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (static_cast<int32_t>(threadIdx.x) < F) {
        double r = part[0] / count;
        if (take_sqrt) r = sqrt(r);
        for (int32_t f = threadIdx.x; f < F; f += kThreads) {
            out64[f] = r;
            out32[f] = static_cast<float>(r);
        }
    }
}

// One workgroup per feature: thread i adds the rows i, i+256, ... in time order, then a fixed
// LDS tree; result / (T*N), optionally square-rooted.
__global__ void __launch_bounds__(kThreads) reduce_rows_kernel(const double* __restrict__ row_acc, int64_t T,
                                                               int32_t N, int32_t F, int take_sqrt,
                                                               double* __restrict__ out64,
                                                               float* __restrict__ out32) {
    __shared__ double part[kThreads];
    const int32_t f = blockIdx.x;
    double acc = 0.0;
    // rows are read eight ahead (one workgroup walks a whole column); the additions keep the row order
    constexpr int kAhead = 8;
    int64_t t = threadIdx.x;
    for (; t + static_cast<int64_t>(kThreads) * (kAhead - 1) < T; t += static_cast<int64_t>(kThreads) * kAhead) {
        double v[kAhead];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) v[u] = row_acc[(t + static_cast<int64_t>(kThreads) * u) * F + f];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) acc += v[u];
    }
    for (; t < T; t += kThreads) acc += row_acc[t * F + f];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (uint32_t off = kThreads / 2; off >= 1; off >>= 1) {
        if (threadIdx.x < off) part[threadIdx.x] += part[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        double r = part[0] / (static_cast<double>(T) * static_cast<double>(N));
        if (take_sqrt) r = sqrt(r);
        out64[f] = r;
        out32[f] = static_cast<float>(r);
    }
}

}  // namespace

hipError_t launch_store_bf16(const float* src, uint16_t* dst, size_t count, hipStream_t s) {
    if (count == 0) return hipSuccess;
    size_t quads = count / 4;
    size_t want = (quads + kThreads - 1) / kThreads;
    uint32_t grid = static_cast<uint32_t>(want < 1 ? 1 : (want > 16384 ? 16384 : want));
    hipLaunchKernelGGL(store_bf16_kernel, dim3(grid), dim3(kThreads), 0, s, src, dst, count);
    return hipGetLastError();
}

hipError_t launch_row_sums(const float* chunk, int64_t rows, int32_t N, int32_t F, int32_t F_src, int32_t period,
                           int64_t row0, const double* mean64, double* row_acc, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int64_t waves = rows * F;
    const int64_t per_block = kThreads / 64;
    const int64_t grid = (waves + per_block - 1) / per_block;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(row_sums_kernel, dim3(static_cast<uint32_t>(grid)), dim3(kThreads), 0, s, chunk, rows,
                       N, F, F_src, period, row0, mean64, row_acc);
    return hipGetLastError();
}

hipError_t launch_reduce_rows(const double* row_acc, int64_t T, int32_t N, int32_t F, bool take_sqrt,
                              double* out64, float* out32, hipStream_t s) {
    hipLaunchKernelGGL(reduce_rows_kernel, dim3(F), dim3(kThreads), 0, s, row_acc, T, N, F,
                       take_sqrt ? 1 : 0, out64, out32);
    return hipGetLastError();
}

hipError_t launch_reduce_rows_alg1(const double* row_acc, int32_t F, int64_t n_train, int32_t P, double count,
                                   bool take_sqrt, double* out64, float* out32, hipStream_t s) {
    hipLaunchKernelGGL(reduce_rows_alg1_kernel, dim3(1), dim3(kThreads), 0, s, row_acc, F, n_train, P, count,
                       take_sqrt ? 1 : 0, out64, out32);
    return hipGetLastError();
}

hipError_t launch_assemble_rows(const float* src, int64_t rows, int32_t N, int32_t F_src, int32_t F, int64_t row0,
                                int32_t period, void* dst, bool out_bf16, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int64_t total = rows * N * F;
    const int64_t want = (total + kThreads - 1) / kThreads;
    const uint32_t grid = static_cast<uint32_t>(want > 65536 ? 65536 : want);
    if (out_bf16)
        hipLaunchKernelGGL(assemble_rows_kernel<true>, dim3(grid), dim3(kThreads), 0, s, src, rows, N, F_src, F, row0,
                           period, dst);
    else
        hipLaunchKernelGGL(assemble_rows_kernel<false>, dim3(grid), dim3(kThreads), 0, s, src, rows, N, F_src, F, row0,
                           period, dst);
    return hipGetLastError();
}

}  // namespace pgti
