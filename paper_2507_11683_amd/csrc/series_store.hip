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

// One wave per (row, feature): lane l adds the nodes l, l+64, ... in node order, then the 64 lane
// sums are combined in a fixed butterfly.  The order depends on nothing but N, so the result does
// not depend on how the series was cut into chunks.
__global__ void __launch_bounds__(kThreads) row_sums_kernel(const float* __restrict__ chunk, int64_t rows,
                                                            int32_t N, int32_t F, int64_t row0,
                                                            const double* __restrict__ mean64,
                                                            double* __restrict__ row_acc) {
    const uint32_t lane = threadIdx.x & 63u;
    const int64_t wave = static_cast<int64_t>(blockIdx.x) * (kThreads / 64) + (threadIdx.x >> 6);
    if (wave >= rows * F) return;  // whole waves leave together
    const int64_t row = wave / F;
    const int32_t f = static_cast<int32_t>(wave % F);
    const float* p = chunk + row * static_cast<int64_t>(N) * F + f;
    const double mu = mean64 ? mean64[f] : 0.0;
    double acc = 0.0;
    for (int32_t node = lane; node < N; node += 64) {
        double v = static_cast<double>(p[static_cast<int64_t>(node) * F]);
        if (mean64) {
            double d = v - mu;
            acc += d * d;
        } else {
            acc += v;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) row_acc[(row0 + row) * F + f] = acc;
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
    for (int64_t t = threadIdx.x; t < T; t += kThreads) acc += row_acc[t * F + f];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int off = kThreads / 2; off >= 1; off >>= 1) {
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

hipError_t launch_row_sums(const float* chunk, int64_t rows, int32_t N, int32_t F, int64_t row0,
                           const double* mean64, double* row_acc, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    const int64_t waves = rows * F;
    const int64_t per_block = kThreads / 64;
    const int64_t grid = (waves + per_block - 1) / per_block;
    if (grid > 0x7FFFFFFF) return hipErrorInvalidValue;
    hipLaunchKernelGGL(row_sums_kernel, dim3(static_cast<uint32_t>(grid)), dim3(kThreads), 0, s, chunk, rows,
                       N, F, row0, mean64, row_acc);
    return hipGetLastError();
}

hipError_t launch_reduce_rows(const double* row_acc, int64_t T, int32_t N, int32_t F, bool take_sqrt,
                              double* out64, float* out32, hipStream_t s) {
    hipLaunchKernelGGL(reduce_rows_kernel, dim3(F), dim3(kThreads), 0, s, row_acc, T, N, F,
                       take_sqrt ? 1 : 0, out64, out32);
    return hipGetLastError();
}

}  // namespace pgti
