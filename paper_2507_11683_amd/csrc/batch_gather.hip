// Batch build: fused gather + standardise (Sec. 4.1 of the paper: a snapshot is rebuilt at run
// time as x = data[start : start+P], y = data[start+P : start+P+Q]; Algorithm 1: (v - mu)/sigma).
//
// Structure of the work: because a timestep row is contiguous ([T, N, F] with R = N*F elements
// per row), the x and y windows of one sample form ONE contiguous source span of (P+Q)*R
// elements starting at element start*R, and it lands in two contiguous destinations, P*R
// elements of out_x[j] followed by Q*R elements of out_y[j].  The kernel is therefore a batched
// streaming copy with a per-feature affine step in registers: HBM-bound, 2 flops per element,
// no contraction, so no MFMA and no LDS (with shuffled starts two samples of a batch almost never
// share a row, so there is nothing to stage).
//
// Bit exactness: (v - mean[f]) / std[f] is one IEEE binary32 subtraction and one correctly
// rounded binary32 division (the compiler's default expansion; this file is built with
// -ffp-contract=off and without fast-math, fp32 denormals on).
#include "pgti_internal.h"

namespace pgti {
namespace {

constexpr int kThreads = 256;

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct GatherArgs {
    const void* series;     // resident [T, R], fp32 or bf16
    const int32_t* starts;  // this batch's starts
    float* out_x;           // [count, P, R]
    float* out_y;           // [count, Q, R]
    int64_t R;
    int32_t last_start;    // n_windows - 1: starts are clamped to [0, last_start] before use
    uint32_t units_x;      // quads (or elements, scalar path) of one sample's x window
    uint32_t units_total;  // ... of the whole (P+Q) span
    uint32_t F;
    float mean[kInlineStats];
    float stdev[kInlineStats];
    const float* d_mean;  // used when F > kInlineStats
    const float* d_std;
};

__device__ __forceinline__ float widen_bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float widen_bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Element offset of sample j's span.  The share holds a permutation of valid starts; the clamp only
// guarantees that no address outside the series can ever be formed.
__device__ __forceinline__ int64_t span_offset(const GatherArgs& a, uint32_t j) {
    int32_t start = a.starts[j];
    start = start < 0 ? 0 : (start > a.last_start ? a.last_start : start);
    return static_cast<int64_t>(start) * a.R;
}

// Loads the 4 consecutive stored elements that start at element offset `e` of the series.
// ALIGN_CLASS 0: e % 4 == 0 (one vector load); 2: e % 4 == 2 (two half loads); 1: odd (four).
template <int STORE_BYTES, int ALIGN_CLASS>
__device__ __forceinline__ f32x4 load_quad(const void* series, int64_t e) {
    f32x4 v;
    if constexpr (STORE_BYTES == 4) {
        const float* p = static_cast<const float*>(series) + e;
        if constexpr (ALIGN_CLASS == 0) {
            v = *reinterpret_cast<const f32x4*>(p);
        } else if constexpr (ALIGN_CLASS == 2) {
            f32x2 a = *reinterpret_cast<const f32x2*>(p);
            f32x2 b = *reinterpret_cast<const f32x2*>(p + 2);
            v = f32x4{a.x, a.y, b.x, b.y};
        } else {
            v = f32x4{p[0], p[1], p[2], p[3]};
        }
    } else {
        const uint16_t* p = static_cast<const uint16_t*>(series) + e;
        if constexpr (ALIGN_CLASS == 0) {
            u32x2 w = *reinterpret_cast<const u32x2*>(p);
            v = f32x4{widen_bf16_lo(w.x), widen_bf16_hi(w.x), widen_bf16_lo(w.y), widen_bf16_hi(w.y)};
        } else if constexpr (ALIGN_CLASS == 2) {
            uint32_t a = *reinterpret_cast<const uint32_t*>(p);
            uint32_t b = *reinterpret_cast<const uint32_t*>(p + 2);
            v = f32x4{widen_bf16_lo(a), widen_bf16_hi(a), widen_bf16_lo(b), widen_bf16_hi(b)};
        } else {
            v = f32x4{widen_bf16_lo(p[0]), widen_bf16_lo(p[1]), widen_bf16_lo(p[2]), widen_bf16_lo(p[3])};
        }
    }
    return v;
}

// (v - mean[f]) / std[f] for the four elements of quad q.  FSTATIC in {1, 2, 4}: the feature of
// lane k of a quad does not depend on q (every span starts on a row, so on feature 0);
// FSTATIC == 0: any F, the feature is ((4q + k) mod F).
template <int FSTATIC>
__device__ __forceinline__ f32x4 standardise_quad(f32x4 v, uint32_t q, const GatherArgs& a) {
    f32x4 m, s;
    if constexpr (FSTATIC == 1) {
        m = f32x4{a.mean[0], a.mean[0], a.mean[0], a.mean[0]};
        s = f32x4{a.stdev[0], a.stdev[0], a.stdev[0], a.stdev[0]};
    } else if constexpr (FSTATIC == 2) {
        m = f32x4{a.mean[0], a.mean[1], a.mean[0], a.mean[1]};
        s = f32x4{a.stdev[0], a.stdev[1], a.stdev[0], a.stdev[1]};
    } else if constexpr (FSTATIC == 4) {
        m = f32x4{a.mean[0], a.mean[1], a.mean[2], a.mean[3]};
        s = f32x4{a.stdev[0], a.stdev[1], a.stdev[2], a.stdev[3]};
    } else {
        uint32_t f0 = static_cast<uint32_t>((4ull * q) % a.F);
        uint32_t f1 = (f0 + 1) % a.F, f2 = (f0 + 2) % a.F, f3 = (f0 + 3) % a.F;
        m = f32x4{a.d_mean[f0], a.d_mean[f1], a.d_mean[f2], a.d_mean[f3]};
        s = f32x4{a.d_std[f0], a.d_std[f1], a.d_std[f2], a.d_std[f3]};
    }
    f32x4 r;
    r.x = (v.x - m.x) / s.x;
    r.y = (v.y - m.y) / s.y;
    r.z = (v.z - m.z) / s.z;
    r.w = (v.w - m.w) / s.w;
    return r;
}

// grid = (ceil(units_total / (kThreads*UNROLL)), count).  Workgroup (bx, j) handles quads
// [bx*kThreads*UNROLL, ...) of sample j; consecutive lanes take consecutive quads, so every load
// and store instruction of a wave covers 1 KiB of contiguous memory.  All UNROLL loads are
// issued before the first use to keep UNROLL*16 bytes per lane in flight.
template <int STORE_BYTES, int FSTATIC, int UNROLL>
__global__ void __launch_bounds__(kThreads) gather_quads_kernel(GatherArgs a) {
    const uint32_t j = blockIdx.y;
    const int64_t e0 = span_offset(a, j);
    const uint32_t q0 = blockIdx.x * (kThreads * UNROLL) + threadIdx.x;
    const uint32_t align = static_cast<uint32_t>(e0) & 3u;  // uniform over the workgroup

    f32x4 v[UNROLL];
    if (align == 0) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            uint32_t q = q0 + u * kThreads;
            if (q < a.units_total) v[u] = load_quad<STORE_BYTES, 0>(a.series, e0 + 4ll * q);
        }
    } else if (align == 2) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            uint32_t q = q0 + u * kThreads;
            if (q < a.units_total) v[u] = load_quad<STORE_BYTES, 2>(a.series, e0 + 4ll * q);
        }
    } else {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            uint32_t q = q0 + u * kThreads;
            if (q < a.units_total) v[u] = load_quad<STORE_BYTES, 1>(a.series, e0 + 4ll * q);
        }
    }

    f32x4* x_base = reinterpret_cast<f32x4*>(a.out_x) + static_cast<size_t>(j) * a.units_x;
    f32x4* y_base = reinterpret_cast<f32x4*>(a.out_y) +
                    static_cast<size_t>(j) * (a.units_total - a.units_x);
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        uint32_t q = q0 + u * kThreads;
        if (q < a.units_total) {
            f32x4 r = standardise_quad<FSTATIC>(v[u], q, a);
            f32x4* dst = (q < a.units_x) ? (x_base + q) : (y_base + (q - a.units_x));
            __builtin_nontemporal_store(r, dst);  // written once, never re-read by this kernel
        }
    }
}

// Any geometry (P*R or Q*R not a multiple of 4): one element per thread.
template <int STORE_BYTES>
__global__ void __launch_bounds__(kThreads) gather_scalar_kernel(GatherArgs a) {
    const uint32_t j = blockIdx.y;
    const int64_t e0 = span_offset(a, j);
    const uint32_t e = blockIdx.x * kThreads + threadIdx.x;
    if (e >= a.units_total) return;
    float v;
    if constexpr (STORE_BYTES == 4) {
        v = static_cast<const float*>(a.series)[e0 + e];
    } else {
        v = widen_bf16_lo(static_cast<const uint16_t*>(a.series)[e0 + e]);
    }
    const uint32_t f = e % a.F;
    const float r = (v - a.d_mean[f]) / a.d_std[f];
    float* dst = (e < a.units_x)
                     ? a.out_x + static_cast<size_t>(j) * a.units_x + e
                     : a.out_y + static_cast<size_t>(j) * (a.units_total - a.units_x) + (e - a.units_x);
    *dst = r;
}

template <int STORE_BYTES, int FSTATIC>
void launch_quads(const GatherArgs& a, int32_t count, hipStream_t s) {
    // Large samples: 8 quads (128 B) per lane in flight.  Small samples: 1 quad per lane so that
    // a sample still spreads over several workgroups.
    if (a.units_total >= 8u * kThreads * 8u) {
        dim3 grid((a.units_total + kThreads * 8 - 1) / (kThreads * 8), count);
        hipLaunchKernelGGL((gather_quads_kernel<STORE_BYTES, FSTATIC, 8>), grid, dim3(kThreads), 0, s, a);
    } else {
        dim3 grid((a.units_total + kThreads - 1) / kThreads, count);
        hipLaunchKernelGGL((gather_quads_kernel<STORE_BYTES, FSTATIC, 1>), grid, dim3(kThreads), 0, s, a);
    }
}

template <int STORE_BYTES>
void launch_quads_f(const GatherArgs& a, int32_t count, hipStream_t s) {
    if (a.F == 1) launch_quads<STORE_BYTES, 1>(a, count, s);
    else if (a.F == 2) launch_quads<STORE_BYTES, 2>(a, count, s);
    else if (a.F == 4) launch_quads<STORE_BYTES, 4>(a, count, s);
    else launch_quads<STORE_BYTES, 0>(a, count, s);
}

}  // namespace

hipError_t launch_batch_gather(const pgti_ctx* c, const int32_t* d_starts, int32_t count,
                               float* out_x, float* out_y, hipStream_t s) {
    GatherArgs a{};
    a.series = c->d_series;
    a.starts = d_starts;
    a.out_x = out_x;
    a.out_y = out_y;
    a.R = c->R;
    a.last_start = static_cast<int32_t>(c->n_windows - 1);
    a.F = static_cast<uint32_t>(c->F);
    for (int f = 0; f < kInlineStats && f < c->F; ++f) {
        a.mean[f] = c->mean[f];
        a.stdev[f] = c->stdev[f];
    }
    a.d_mean = c->d_stats;
    a.d_std = c->d_stats + c->F;
    const int64_t ex = static_cast<int64_t>(c->P) * c->R, et = static_cast<int64_t>(c->P + c->Q) * c->R;
    if (c->path == GatherPath::kQuads) {
        a.units_x = static_cast<uint32_t>(ex / 4);
        a.units_total = static_cast<uint32_t>(et / 4);
        if (c->storage == PGTI_F32) launch_quads_f<4>(a, count, s);
        else launch_quads_f<2>(a, count, s);
    } else {
        a.units_x = static_cast<uint32_t>(ex);
        a.units_total = static_cast<uint32_t>(et);
        dim3 grid((a.units_total + kThreads - 1) / kThreads, count);
        if (c->storage == PGTI_F32)
            hipLaunchKernelGGL((gather_scalar_kernel<4>), grid, dim3(kThreads), 0, s, a);
        else
            hipLaunchKernelGGL((gather_scalar_kernel<2>), grid, dim3(kThreads), 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace pgti
