// Resident series store (Sec. 4.1 of the paper, GPU-Index-Batching: the data is migrated to GPU
// memory once and the preprocessing runs there; Eq. 2: a single copy of the data is kept).
// Device-side work of a load, all in one streaming kernel per chunk of rows:
//   * writing the resident rows: plain fp32, or rounded to bf16, optionally with the time-of-day
//     feature appended to every node (stage 1 of the preprocessing);
//   * the row sums behind the statistics (Algorithm 1 standardises with a mean and a standard
//     deviation): per (row, feature) the fp64 sum of the values, or of the squared deviations from a
//     given mean, taken over the nodes IN NODE ORDER, one addition after the other.  The order is
//     part of the definition of the statistics (row by row, then the row sums in time order), so the
//     result does not depend on the launch shape and equals a plain sequential loop bit for bit.
//
// How a sequential sum runs at memory speed: a workgroup owns up to 32 rows and walks them tile by
// tile (32 rows x 256 columns).  All 256 lanes load the tile with coalesced 16-byte accesses (and
// store it to the resident series on the way); the tile goes to LDS; then one lane per (row,
// feature) chain adds its elements of the tile to its running fp64 sum, in order.  The next tile's
// loads are issued before that serial phase, and several workgroups share a CU, so memory stays
// busy while the chains advance.  105,120 rows x 2 features give 210,240 independent chains.
// A step of a chain costs a SIMD about 48 cycles whether 2 or 64 lanes of the wave take part, so the
// tile is as tall as the 64 KB of LDS allow with rows of 1 KB: 64 chains per serial phase keep the
// sums (and, measured, the whole kernel: it runs as fast with the sums switched off) memory bound.
// Wider, shorter tiles stream a little faster (8 x 1024: +6 %) but their 16 chains become the limit.
#include <type_traits>

#include "pgti_internal.h"

namespace pgti {
namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = 32;
constexpr int kTileCols = 256;
constexpr int kTilePitchMax = kTileCols + 31;
constexpr int kGroupFeatures = 256;  // chains of one workgroup cover at most this many features

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Round to nearest, ties to even, on the upper 16 bits.  NaN keeps sign and upper payload and
// gets the quiet bit so that it cannot round to infinity.
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Time of day of absolute timestep t: (t mod period) / period, the quotient taken in binary32.
__device__ __forceinline__ float time_of_day(int64_t t, int32_t period) {
    return static_cast<float>(static_cast<int32_t>(t % period)) / static_cast<float>(period);
}

struct IngestArgs {
    const float* src;      // [rows][N * F_src] fp32
    void* dst;             // [rows][N * F] fp32 or bf16 (dst_bf16), or null: nothing is written
    const double* mean64;  // null: sums of values; else sums of squared deviations from mean64[f]
    double* row_acc;       // [all rows of the series][F], or null: no sums
    int64_t rows;          // rows of this chunk
    int64_t row0;          // absolute index of the chunk's first row
    int32_t N, F, F_src, period;
    int32_t rows_blk;      // rows per workgroup: rows_blk * min(F, 256) <= 256
    int32_t dst_bf16;
};

// One chain's share of a tile: acc = (...((acc + t(x_j)) + t(x_{j+F})) + ...) over the elements
// j, j+F, j+2F, ... < width of an LDS row, in that order; t(x) = x widened to fp64, or its squared
// deviation from mu (two roundings: the subtraction and the product).  The additions are serial by
// definition; the LDS reads of the next eight elements are issued before the current eight are
// added.
template <bool SQUARES>
__device__ __forceinline__ double fold_chain(const float* __restrict__ rowp, int32_t j, int32_t width, int32_t F,
                                             double mu, double acc) {
    constexpr int kBurst = 8;
    auto term = [&](float x) -> double {
        if constexpr (SQUARES) {
            const double d = static_cast<double>(x) - mu;
            return d * d;
        } else {
            return static_cast<double>(x);
        }
    };
    const int32_t step = kBurst * F, reach = (kBurst - 1) * F;
    if (j + reach < width) {
        float cur[kBurst], nxt[kBurst];
#pragma unroll
        for (int u = 0; u < kBurst; ++u) cur[u] = rowp[j + u * F];
        j += step;
        while (j + reach < width) {
#pragma unroll
            for (int u = 0; u < kBurst; ++u) nxt[u] = rowp[j + u * F];
#pragma unroll
            for (int u = 0; u < kBurst; ++u) acc += term(cur[u]);
#pragma unroll
            for (int u = 0; u < kBurst; ++u) cur[u] = nxt[u];
            j += step;
        }
#pragma unroll
        for (int u = 0; u < kBurst; ++u) acc += term(cur[u]);
    }
    for (; j < width; j += F) acc += term(rowp[j]);
    return acc;
}

// VEC4: a lane moves 16-byte quads of the OUTPUT row (rows are whole quads and the pointers are
// aligned for them); SYNTH: F_src = F - 1 and feature F - 1 is the time of day of the row.  VEC4 with
// SYNTH is the common case of one stored feature plus the time of day (F_src = 1, F = 2): an output
// quad is (v0, tod, v1, tod), made from one 8-byte load.
template <bool VEC4, bool SYNTH>
__global__ void __launch_bounds__(kThreads) ingest_rows_kernel(IngestArgs a) {
    __shared__ float tile[kTileRows * kTilePitchMax];
    __shared__ float tods[kTileRows];  // time of day of the workgroup's rows (SYNTH)
    using Reg = typename std::conditional<VEC4, f32x4, float>::type;
    constexpr int kPasses = VEC4 ? (kTileRows * kTileCols / 4) / kThreads : kTileRows;

    const uint32_t tid = threadIdx.x;
    const int32_t F = a.F;
    const int64_t R = static_cast<int64_t>(a.N) * F, R_src = static_cast<int64_t>(a.N) * a.F_src;
    const int64_t r_first = static_cast<int64_t>(blockIdx.x) * a.rows_blk;  // inside the chunk
    const int64_t rows_left = a.rows - r_first;
    const int32_t rows_here = rows_left < a.rows_blk ? static_cast<int32_t>(rows_left) : a.rows_blk;
    const int32_t f_lo = static_cast<int32_t>(blockIdx.y) * kGroupFeatures;
    const int32_t Fg = (F - f_lo < kGroupFeatures) ? F - f_lo : kGroupFeatures;
    const uint32_t pitch = kTileCols + (F & 31);  // chain c reads bank (c + const) mod 32: no conflicts
    const bool sums = a.row_acc != nullptr;
    const bool squares = a.mean64 != nullptr;
    const bool writes = a.dst != nullptr && blockIdx.y == 0;
    const bool has_chain = sums && static_cast<int32_t>(tid) < rows_here * Fg;
    const int32_t chain_row = static_cast<int32_t>(tid) / Fg, chain_f = f_lo + static_cast<int32_t>(tid) % Fg;
    double acc = 0.0;
    const double mu = (has_chain && squares) ? a.mean64[chain_f] : 0.0;

    // position of this lane's element(s) inside a tile: pass p takes quad p*256 + tid of the tile (VEC4)
    // or element tid of row p
    auto pass_row = [&](int p) -> int32_t {
        return VEC4 ? static_cast<int32_t>((p * kThreads + tid) / (kTileCols / 4)) : p;
    };
    auto pass_col = [&](int p) -> int32_t {
        return VEC4 ? 4 * static_cast<int32_t>((p * kThreads + tid) % (kTileCols / 4)) : static_cast<int32_t>(tid);
    };

    if constexpr (SYNTH) {
        if (tid < kTileRows) tods[tid] = time_of_day(a.row0 + r_first + tid, a.period);
        __syncthreads();
    }

    Reg regs[kPasses];
    auto load_tile = [&](int64_t c0) {
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int32_t rr = pass_row(p), lane_col = pass_col(p);
            const int64_t col = c0 + lane_col;
            const bool valid = rr < rows_here && col < R;
            if constexpr (VEC4 && SYNTH) {
                regs[p] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (valid) {
                    const u32x2* sp = reinterpret_cast<const u32x2*>(a.src + (r_first + rr) * R_src + (col >> 1));
                    const u32x2 v = __builtin_nontemporal_load(sp);
                    const float tod = tods[rr];
                    regs[p] = f32x4{__uint_as_float(v.x), tod, __uint_as_float(v.y), tod};
                }
            } else if constexpr (VEC4) {
                regs[p] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (valid) {
                    const f32x4* sp = reinterpret_cast<const f32x4*>(a.src + (r_first + rr) * R + col);
                    regs[p] = __builtin_nontemporal_load(sp);  // every byte is used once
                }
            } else if constexpr (SYNTH) {
                regs[p] = 0.f;
                if (valid) {
                    const int32_t node = static_cast<int32_t>(col) / F, f = static_cast<int32_t>(col) - node * F;
                    regs[p] = (f < a.F_src) ? a.src[(r_first + rr) * R_src + static_cast<int64_t>(node) * a.F_src + f]
                                            : tods[rr];
                }
            } else {
                regs[p] = 0.f;
                if (valid) regs[p] = a.src[(r_first + rr) * R + col];
            }
        }
    };

    load_tile(0);
    for (int64_t c0 = 0; c0 < R; c0 += kTileCols) {
        // registers -> resident series, registers -> LDS
#pragma unroll
        for (int p = 0; p < kPasses; ++p) {
            const int32_t rr = pass_row(p), lane_col = pass_col(p);
            const int64_t col = c0 + lane_col;
            const bool valid = rr < rows_here && col < R;
            if (writes && valid) {
                const int64_t at = (r_first + rr) * R + col;
                if constexpr (VEC4) {
                    if (a.dst_bf16) {
                        u32x2 o;
                        o.x = bf16_bits(regs[p].x) | (bf16_bits(regs[p].y) << 16);
                        o.y = bf16_bits(regs[p].z) | (bf16_bits(regs[p].w) << 16);
                        u32x2* dp = reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.dst) + at);
                        __builtin_nontemporal_store(o, dp);
                    } else {
                        f32x4* dp = reinterpret_cast<f32x4*>(static_cast<float*>(a.dst) + at);
                        __builtin_nontemporal_store(regs[p], dp);
                    }
                } else {
                    if (a.dst_bf16) static_cast<uint16_t*>(a.dst)[at] = static_cast<uint16_t>(bf16_bits(regs[p]));
                    else static_cast<float*>(a.dst)[at] = regs[p];
                }
            }
            if (sums) {
                float* t = tile + rr * pitch + lane_col;
                if constexpr (VEC4) {
                    t[0] = regs[p].x;
                    t[1] = regs[p].y;
                    t[2] = regs[p].z;
                    t[3] = regs[p].w;
                } else {
                    t[0] = regs[p];
                }
            }
        }
        if (!sums) {
            if (c0 + kTileCols < R) load_tile(c0 + kTileCols);
            continue;
        }
        __syncthreads();
        if (c0 + kTileCols < R) load_tile(c0 + kTileCols);  // in flight during the serial phase
        if (has_chain) {
            const int32_t width = (R - c0 < kTileCols) ? static_cast<int32_t>(R - c0) : kTileCols;
            const int32_t phase = static_cast<int32_t>(c0) % F;
            int32_t j = chain_f - phase;  // first column of the tile that holds feature chain_f
            if (j < 0) j += F;
            const float* rowp = tile + chain_row * pitch;
            acc = squares ? fold_chain<true>(rowp, j, width, F, mu, acc) : fold_chain<false>(rowp, j, width, F, mu, acc);
        }
        __syncthreads();
    }
    if (has_chain) a.row_acc[(a.row0 + r_first + chain_row) * F + chain_f] = acc;
}

// The row sums in time order: thread f of workgroup b adds row_acc[t][256 b + f] for t = 0, 1, ...
// T-1, one after the other (the order is part of the definition).  All lanes stage the table through
// LDS, 2,048 entries at a time and transposed, so that every chain finds its values side by side; the
// next chunk's loads are in flight while the chains advance, and a chain fetches its next sixteen values
// from LDS while it adds the current sixteen, so that only the additions themselves are serial.
// result = total / count, optionally square-rooted; out64 keeps it for the next sweep.
constexpr int kReduceChunk = 2048;

__global__ void __launch_bounds__(kThreads) reduce_rows_seq_kernel(const double* __restrict__ row_acc, int64_t T,
                                                                   int32_t F, double count, int take_sqrt,
                                                                   double* __restrict__ out64,
                                                                   float* __restrict__ out32) {
    __shared__ double buf[kReduceChunk];
    constexpr int kPer = kReduceChunk / kThreads;
    constexpr int kBurst = 16;
    const int32_t tid = threadIdx.x;
    const int32_t f0 = static_cast<int32_t>(blockIdx.x) * kGroupFeatures;
    const int32_t Fb = (F - f0 < kGroupFeatures) ? F - f0 : kGroupFeatures;
    const int32_t rows_chunk = kReduceChunk / Fb;  // >= 8
    double regs[kPer];
    auto load_chunk = [&](int64_t t0) {
        const int64_t rows = (T - t0 < rows_chunk) ? T - t0 : rows_chunk;
#pragma unroll
        for (int p = 0; p < kPer; ++p) {
            const int32_t idx = tid + p * kThreads;
            const int32_t r = idx / Fb, fl = idx - r * Fb;
            regs[p] = (r < rows) ? row_acc[(t0 + r) * F + f0 + fl] : 0.0;
        }
    };
    double total = 0.0;
    load_chunk(0);
    for (int64_t t0 = 0; t0 < T; t0 += rows_chunk) {
#pragma unroll
        for (int p = 0; p < kPer; ++p) {
            const int32_t idx = tid + p * kThreads;
            const int32_t r = idx / Fb, fl = idx - r * Fb;
            if (r < rows_chunk) buf[fl * rows_chunk + r] = regs[p];
        }
        __syncthreads();
        if (t0 + rows_chunk < T) load_chunk(t0 + rows_chunk);
        if (tid < Fb) {
            const int32_t rows = static_cast<int32_t>((T - t0 < rows_chunk) ? T - t0 : rows_chunk);
            const double* mine = buf + tid * rows_chunk;
            // two register buffers take turns: while one burst is added, the next is on its way from LDS
            double va[kBurst], vb[kBurst];
            auto fetch = [&](double (&v)[kBurst], int32_t at) {
#pragma unroll
                for (int u = 0; u < kBurst; ++u) v[u] = mine[at + u];
            };
            auto add_all = [&](const double (&v)[kBurst]) {
#pragma unroll
                for (int u = 0; u < kBurst; ++u) total += v[u];
            };
            int32_t r = 0;
            if (rows >= kBurst) {
                fetch(va, 0);
                r = kBurst;
                while (r + 2 * kBurst <= rows) {
                    fetch(vb, r);
                    add_all(va);
                    fetch(va, r + kBurst);
                    add_all(vb);
                    r += 2 * kBurst;
                }
                add_all(va);
            }
            for (; r < rows; ++r) total += mine[r];
        }
        __syncthreads();
    }
    if (tid < Fb) {
        double r = total / count;
        if (take_sqrt) r = sqrt(r);
        out64[f0 + tid] = r;
        out32[f0 + tid] = static_cast<float>(r);
    }
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

}  // namespace

hipError_t launch_ingest_rows(const float* src, int64_t rows, int32_t N, int32_t F, int32_t F_src, int32_t period,
                              int64_t row0, void* dst, bool dst_bf16, const double* mean64, double* row_acc,
                              hipStream_t s) {
    if (rows <= 0 || (!dst && !row_acc)) return hipSuccess;
    if (F_src != F && (F_src != F - 1 || period <= 0)) return hipErrorInvalidValue;
    IngestArgs a{};
    a.src = src;
    a.dst = dst;
    a.mean64 = mean64;
    a.row_acc = row_acc;
    a.rows = rows;
    a.row0 = row0;
    a.N = N;
    a.F = F;
    a.F_src = F_src;
    a.period = period;
    a.dst_bf16 = dst_bf16 ? 1 : 0;
    const int32_t Fg = F < kGroupFeatures ? F : kGroupFeatures;
    a.rows_blk = kThreads / Fg < kTileRows ? kThreads / Fg : kTileRows;
    const int64_t blocks = (rows + a.rows_blk - 1) / a.rows_blk;
    const int64_t groups = row_acc ? (F + kGroupFeatures - 1) / kGroupFeatures : 1;
    if (blocks > 0x7FFFFFFF || groups > 65535) return hipErrorInvalidValue;
    const dim3 grid(static_cast<uint32_t>(blocks), static_cast<uint32_t>(groups)), block(kThreads);
    const int64_t R = static_cast<int64_t>(N) * F;
    const bool synth = F_src != F;
    const uintptr_t dst_align = dst ? reinterpret_cast<uintptr_t>(dst) & (dst_bf16 ? 7u : 15u) : 0u;
    const bool vec4 = !synth && R % 4 == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0 && dst_align == 0;
    const bool synth_pairs = synth && F == 2 && N % 2 == 0 && (reinterpret_cast<uintptr_t>(src) & 7u) == 0 && dst_align == 0;
    if (synth_pairs) hipLaunchKernelGGL((ingest_rows_kernel<true, true>), grid, block, 0, s, a);
    else if (synth) hipLaunchKernelGGL((ingest_rows_kernel<false, true>), grid, block, 0, s, a);
    else if (vec4) hipLaunchKernelGGL((ingest_rows_kernel<true, false>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((ingest_rows_kernel<false, false>), grid, block, 0, s, a);
    return hipGetLastError();
}

hipError_t launch_reduce_rows(const double* row_acc, int64_t T, int32_t N, int32_t F, bool take_sqrt,
                              double* out64, float* out32, hipStream_t s) {
    const uint32_t blocks = static_cast<uint32_t>((F + kGroupFeatures - 1) / kGroupFeatures);
    hipLaunchKernelGGL(reduce_rows_seq_kernel, dim3(blocks), dim3(kThreads), 0, s, row_acc, T, F,
                       static_cast<double>(T) * static_cast<double>(N), take_sqrt ? 1 : 0, out64, out32);
    return hipGetLastError();
}

hipError_t launch_reduce_rows_alg1(const double* row_acc, int32_t F, int64_t n_train, int32_t P, double count,
                                   bool take_sqrt, double* out64, float* out32, hipStream_t s) {
    hipLaunchKernelGGL(reduce_rows_alg1_kernel, dim3(1), dim3(kThreads), 0, s, row_acc, F, n_train, P, count,
                       take_sqrt ? 1 : 0, out64, out32);
    return hipGetLastError();
}

}  // namespace pgti
