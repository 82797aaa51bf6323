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
// Bit exactness: (v - mean[f]) / std[f] is one IEEE binary32 subtraction followed by a correctly
// rounded binary32 division.  The division has two implementations with identical results:
//   * the compiler's expansion of `/` (this file is built with -ffp-contract=off, no fast-math,
//     fp32 denormals on), used whenever a guard fails;
//   * a fast path: the divisor is one of F constants, so its reciprocal r = RN(1/sigma) is
//     computed once on the host (in fp64, rounded once), and q0 = d*r is corrected twice with
//     the exact residual, e = fma(-sigma, q, d); q = fma(e, r, q).  The second correction applied
//     to a faithful quotient with a correctly rounded reciprocal yields RN(d/sigma) (Markstein's
//     theorem) as long as nothing overflows or underflows.  With sigma's biased exponent in
//     [95, 159] (checked once on the host) a resulting quotient whose exponent lies in [96, 158]
//     implies a dividend for which that held, so the result is accepted on that test alone and
//     everything else (zeros, subnormals, infinities, NaNs, extreme magnitudes) is divided again
//     with `/`.  6 full-rate VALU operations per element instead of
//     about 15 issue slots; it matters when the stored type is bf16 (+4 points of the HBM peak) and is
//     hidden behind memory time for fp32.  tests/fastdiv_model.c checks the identity on the host
//     for all 2^32 dividends of hard divisors and for random divisors.
#include <type_traits>

#include "pgti_internal.h"

namespace pgti {
namespace {

constexpr int kThreads = 256;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));       // element-aligned quad
typedef uint32_t u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));    // four bf16, element aligned

struct GatherArgs {
    const void* series;     // resident [T, R], fp32 or bf16
    const int32_t* starts;  // this batch's starts
    void* out_x;            // [count, P, R], fp32 or bf16
    void* out_y;            // [count, Q, R]
    int64_t R;
    int32_t last_start;    // n_windows - 1: starts are clamped to [0, last_start] before use
    uint32_t units_x;      // quads (or elements, scalar path) of one sample's x window
    uint32_t units_total;  // ... of the whole (P+Q) span
    uint32_t F;
    float mean[kInlineStats];
    float stdev[kInlineStats];
    float recip[kInlineStats];  // RN(1 / stdev[f]), meaningful on the fast-division path only
    const float* d_mean;        // used when F is not 1, 2 or 4
    const float* d_std;
    const float* d_recip;
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

// Loads the 4 consecutive stored elements that start at element offset `e` of the series as one
// vector access.  A span starts at start*R elements, so it is only element aligned in general
// (R = 414 floats: 8 bytes; R = 319: 4 bytes); global memory on gfx950 serves such vector loads,
// hence the under-aligned vector types.  STREAM adds the non-temporal hint: the series is far
// larger than the caches and every byte is used once per launch.
template <int STORE_BYTES, bool STREAM>
__device__ __forceinline__ f32x4 load_quad(const void* series, int64_t e) {
    if constexpr (STORE_BYTES == 4) {
        const f32x4_a4* p = reinterpret_cast<const f32x4_a4*>(static_cast<const float*>(series) + e);
        return STREAM ? __builtin_nontemporal_load(p) : *p;
    } else {
        const u32x2_a2* p = reinterpret_cast<const u32x2_a2*>(static_cast<const uint16_t*>(series) + e);
        const u32x2_a2 w = STREAM ? __builtin_nontemporal_load(p) : *p;
        return f32x4{widen_bf16_lo(w.x), widen_bf16_hi(w.x), widen_bf16_lo(w.y), widen_bf16_hi(w.y)};
    }
}

// d / sigma, correctly rounded.  FAST: reciprocal multiply plus two exact-residual corrections,
// accepted when the quotient's exponent is in the mid range, the ordinary division otherwise (see
// the file header).
__device__ __forceinline__ uint32_t magnitude_bits(float d) { return __float_as_uint(d) & 0x7FFFFFFFu; }

// True when all four quotients have a biased exponent in [96, 158]: the smallest and the largest
// magnitude bit pattern bound all four (NaN and Inf patterns are the largest, zero and subnormals
// the smallest).
__device__ __forceinline__ bool quotients_accepted(f32x4 q) {
    const uint32_t a = magnitude_bits(q.x), b = magnitude_bits(q.y), c = magnitude_bits(q.z),
                   e = magnitude_bits(q.w);
    const uint32_t lo = min(min(a, b), min(c, e));
    const uint32_t hi = max(max(a, b), max(c, e));
    return static_cast<bool>(static_cast<int>(lo >= (96u << 23)) & static_cast<int>(hi < (159u << 23)));
}

__device__ __forceinline__ float corrected_quotient(float d, float sigma, float r) {
    const float q0 = d * r;
    const float e0 = __builtin_fmaf(-sigma, q0, d);
    const float q1 = __builtin_fmaf(e0, r, q0);
    const float e1 = __builtin_fmaf(-sigma, q1, d);
    return __builtin_fmaf(e1, r, q1);
}

// Per-quad constants: mean, std and reciprocal of the feature of each of the four elements.
struct QuadStats {
    f32x4 m, s, r;
};

// FSTATIC in {1, 2, 4}: the feature of element k of a quad does not depend on q (every span
// starts on a row, so on feature 0) and the constants come straight from the argument block;
// FSTATIC == 0: any F, the feature is ((4q + k) mod F) and the constants are read from memory.
template <int FSTATIC, bool FAST>
__device__ __forceinline__ QuadStats quad_stats(uint32_t q, const GatherArgs& a) {
    QuadStats t;
    t.r = f32x4{1.f, 1.f, 1.f, 1.f};
    if constexpr (FSTATIC == 1) {
        t.m = f32x4{a.mean[0], a.mean[0], a.mean[0], a.mean[0]};
        t.s = f32x4{a.stdev[0], a.stdev[0], a.stdev[0], a.stdev[0]};
        if constexpr (FAST) t.r = f32x4{a.recip[0], a.recip[0], a.recip[0], a.recip[0]};
    } else if constexpr (FSTATIC == 2) {
        t.m = f32x4{a.mean[0], a.mean[1], a.mean[0], a.mean[1]};
        t.s = f32x4{a.stdev[0], a.stdev[1], a.stdev[0], a.stdev[1]};
        if constexpr (FAST) t.r = f32x4{a.recip[0], a.recip[1], a.recip[0], a.recip[1]};
    } else if constexpr (FSTATIC == 4) {
        t.m = f32x4{a.mean[0], a.mean[1], a.mean[2], a.mean[3]};
        t.s = f32x4{a.stdev[0], a.stdev[1], a.stdev[2], a.stdev[3]};
        if constexpr (FAST) t.r = f32x4{a.recip[0], a.recip[1], a.recip[2], a.recip[3]};
    } else {
        uint32_t f0 = static_cast<uint32_t>((4ull * q) % a.F);
        uint32_t f1 = (f0 + 1) % a.F, f2 = (f0 + 2) % a.F, f3 = (f0 + 3) % a.F;
        t.m = f32x4{a.d_mean[f0], a.d_mean[f1], a.d_mean[f2], a.d_mean[f3]};
        t.s = f32x4{a.d_std[f0], a.d_std[f1], a.d_std[f2], a.d_std[f3]};
        if constexpr (FAST) t.r = f32x4{a.d_recip[f0], a.d_recip[f1], a.d_recip[f2], a.d_recip[f3]};
    }
    return t;
}

// Keeps the argument-block constants live in scalar registers from this point on, so that their
// (scalar) loads are issued together at the top of the kernel instead of one by one after the data
// has arrived: a wave only lives for one quad, so every serialised load latency costs bandwidth.
template <int FSTATIC>
__device__ __forceinline__ void pin_uniform(const QuadStats& t) {
    if constexpr (FSTATIC == 1) {
        asm volatile("" ::"s"(t.m.x), "s"(t.s.x), "s"(t.r.x));
    } else if constexpr (FSTATIC == 2) {
        asm volatile("" ::"s"(t.m.x), "s"(t.s.x), "s"(t.r.x), "s"(t.m.y), "s"(t.s.y), "s"(t.r.y));
    } else if constexpr (FSTATIC == 4) {
        asm volatile("" ::"s"(t.m.x), "s"(t.s.x), "s"(t.r.x), "s"(t.m.y), "s"(t.s.y), "s"(t.r.y));
        asm volatile("" ::"s"(t.m.z), "s"(t.s.z), "s"(t.r.z), "s"(t.m.w), "s"(t.s.w), "s"(t.r.w));
    }
}

// (v - mean[f]) / std[f] for the four elements of a quad.
template <bool FAST>
__device__ __forceinline__ f32x4 standardise_quad(f32x4 v, const QuadStats& t) {
    const f32x4 d = f32x4{v.x - t.m.x, v.y - t.m.y, v.z - t.m.z, v.w - t.m.w};
    f32x4 o;
    if constexpr (FAST) {
        o.x = corrected_quotient(d.x, t.s.x, t.r.x);
        o.y = corrected_quotient(d.y, t.s.y, t.r.y);
        o.z = corrected_quotient(d.z, t.s.z, t.r.z);
        o.w = corrected_quotient(d.w, t.s.w, t.r.w);
        if (quotients_accepted(o)) return o;  // almost always; the test is off the arithmetic's critical path
    }
    o.x = d.x / t.s.x;
    o.y = d.y / t.s.y;
    o.z = d.z / t.s.z;
    o.w = d.w / t.s.w;
    return o;
}

// grid = (ceil(units_total / THREADS), count): workgroup (bx, j) handles THREADS consecutive
// quads of sample j, one quad per lane, so each load and each store instruction of a wave covers
// 1 KiB of contiguous memory.  One quad per lane with many resident waves measured faster on
// MI355X than deeper per-lane unrolling (more, shorter waves keep both the read and the write
// stream busy); the division costs nothing at this rate.
// fp32 -> bf16, round to nearest even on the upper 16 bits; NaN keeps sign and upper payload and
// gets the quiet bit (same rule as the bf16 storage rounding).
__device__ __forceinline__ uint32_t bf16_bits(float v) {
    const uint32_t u = __float_as_uint(v);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// Output stores carry the non-temporal hint (written once, never re-read by these kernels).  With
// fp32 storage they also carry agent scope: on MI355X `sc1 nt` stores measured 3.5 % faster than `nt`
// alone for the 1:1 read-stream + write-stream mix (80.3 % vs 77.6 % of the HBM peak in the same
// harness), plain stores 71 %; with bf16 storage (1:2 mix) `nt` alone measured 0.5 % faster.  The
// compiler's non-temporal builtin only sets `nt`, hence the asm statements.
template <bool AGENT_SCOPE>
__device__ __forceinline__ void stream_store_16(void* dst, f32x4 v) {
    if constexpr (AGENT_SCOPE) asm volatile("global_store_dwordx4 %0, %1, off sc1 nt" ::"v"(dst), "v"(v) : "memory");
    else asm volatile("global_store_dwordx4 %0, %1, off nt" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void stream_store_8(void* dst, u32x2 v) {
    asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" ::"v"(dst), "v"(v) : "memory");
}

// Where output quad q of sample j goes: 16 bytes of fp32, or 8 bytes when the outputs are bf16.
// Computed (and anchored in registers) before the loaded data is needed, so that the address
// arithmetic runs while the load is in flight: a wave lives for one quad, and every instruction
// between the arrival of its data and its store costs bandwidth (+2 points with bf16 storage).
template <bool OUT_BF16>
__device__ __forceinline__ void* quad_destination(const GatherArgs& a, uint32_t j, uint32_t q) {
    constexpr size_t kBytes = OUT_BF16 ? 8 : 16;
    const bool in_x = q < a.units_x;
    char* base = static_cast<char*>(in_x ? a.out_x : a.out_y);
    const size_t index = in_x ? static_cast<size_t>(j) * a.units_x + q
                              : static_cast<size_t>(j) * (a.units_total - a.units_x) + (q - a.units_x);
    void* dst = base + index * kBytes;
    asm volatile("" ::"v"(dst));
    return dst;
}

// Stores one standardised quad at dst: fp32, or bf16 (round to nearest even).
template <bool OUT_BF16, bool AGENT_SCOPE>
__device__ __forceinline__ void store_quad(void* dst, f32x4 r) {
    if constexpr (OUT_BF16) {
        u32x2 o;
        o.x = bf16_bits(r.x) | (bf16_bits(r.y) << 16);
        o.y = bf16_bits(r.z) | (bf16_bits(r.w) << 16);
        stream_store_8(dst, o);
    } else {
        stream_store_16<AGENT_SCOPE>(dst, r);
    }
}

template <int STORE_BYTES, int FSTATIC, int THREADS, bool STREAM, bool FAST, bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gather_quads_kernel(GatherArgs a) {
    const uint32_t j = blockIdx.y;
    const uint32_t q = blockIdx.x * THREADS + threadIdx.x;
    // The start is read before the pin below: an asm statement counts as a possible memory clobber,
    // after which this uniform read would no longer be done by the scalar unit.
    const int64_t e0 = span_offset(a, j);
    const QuadStats t = quad_stats<FSTATIC, FAST>(q, a);
    pin_uniform<FSTATIC>(t);
    if (q >= a.units_total) return;
    const f32x4 v = load_quad<STORE_BYTES, STREAM>(a.series, e0 + 4ll * q);
    void* dst = quad_destination<OUT_BF16>(a, j, q);
    store_quad<OUT_BF16, STORE_BYTES == 4>(dst, standardise_quad<FAST>(v, t));
}

// Row-centric variant for batches of CONSECUTIVE starts (sequential and batch-level-shuffled
// orders): a batch of B' starts s0 .. s0+B'-1 touches only the B'+P+Q-1 source rows
// s0 .. s0+B'+P+Q-2, but each interior row appears in P+Q different (sample, step) slots.
// grid = (ceil(row_quads / THREADS), B+P+Q-1, batches): workgroup (bx, rr, b) loads one chunk of
// source row s0_b + rr ONCE, standardises it once, and stores it to every slot that references
// it: sample j = rr - p for each step p in [0, P+Q) with 0 <= j < B'.  HBM reads drop from
// B'*(P+Q) rows to B'+P+Q-1 rows per batch and the arithmetic by the same factor; the kernel is
// bound by the write stream alone.  Needs rows that start on a quad boundary (R % 4 == 0).
struct RowArgs {
    GatherArgs g;          // units_x / units_total are unused here
    uint32_t B;            // batch size: samples per run
    uint32_t count;        // samples in this launch (the last run may be short)
    uint32_t P, PQ;        // input steps, P + Q
    uint32_t row_quads;    // R / 4
};

template <int STORE_BYTES, int FSTATIC, int THREADS, bool STREAM, bool FAST, bool OUT_BF16>
__global__ void __launch_bounds__(THREADS) gather_rows_kernel(RowArgs a) {
    const uint32_t run = blockIdx.z, rr = blockIdx.y;
    const uint32_t q = blockIdx.x * THREADS + threadIdx.x;  // quad inside the row
    const uint32_t first_sample = run * a.B;
    const uint32_t run_len = min(a.B, a.count - first_sample);
    // First start of the run, clamped so that every row of the run lies inside the series.
    int32_t s0 = a.g.starts[first_sample];
    const int32_t s0_max = a.g.last_start - static_cast<int32_t>(run_len - 1);
    s0 = s0 < 0 ? 0 : (s0 > s0_max ? s0_max : s0);
    const QuadStats t = quad_stats<FSTATIC, FAST>(q, a.g);
    pin_uniform<FSTATIC>(t);
    if (rr >= run_len + a.PQ - 1 || q >= a.row_quads) return;

    const int64_t e = (static_cast<int64_t>(s0) + rr) * a.g.R + 4ll * q;
    const f32x4 r = standardise_quad<FAST>(load_quad<STORE_BYTES, STREAM>(a.g.series, e), t);

    const uint32_t j_lo = (rr >= a.PQ - 1) ? rr - (a.PQ - 1) : 0u;
    const uint32_t j_hi = (rr < run_len - 1) ? rr : run_len - 1;
    const uint32_t Q = a.PQ - a.P;
    for (uint32_t j = j_lo; j <= j_hi; ++j) {
        const uint32_t p = rr - j;  // step of sample j that shows this row
        const size_t sample = first_sample + j;
        constexpr size_t kBytes = OUT_BF16 ? 8 : 16;
        char* dst = (p < a.P) ? static_cast<char*>(a.g.out_x) + ((sample * a.P + p) * a.row_quads + q) * kBytes
                              : static_cast<char*>(a.g.out_y) + ((sample * Q + (p - a.P)) * a.row_quads + q) * kBytes;
        store_quad<OUT_BF16, true>(dst, r);
    }
}

// bf16 storage AND bf16 outputs: a lane with one quad would move only 8 bytes each way and the
// kernel becomes bound by the number of waves, not by memory.  Here a lane takes 8 consecutive
// elements ("oct"): one 16-byte load, one 16-byte store.  Needs P*R and Q*R (span kernel) or R (row
// kernel) to be multiples of 8.  The feature pattern of the second quad equals the first for
// F in {1, 2, 4}; for other F it is looked up again.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_a2 __attribute__((ext_vector_type(4), aligned(2)));

template <int FSTATIC, bool STREAM, bool FAST>
__device__ __forceinline__ u32x4 standardised_oct(const void* series, int64_t e, uint32_t oct, const QuadStats& t,
                                                  const GatherArgs& a) {
    const u32x4_a2* p = reinterpret_cast<const u32x4_a2*>(static_cast<const uint16_t*>(series) + e);
    const u32x4_a2 w = STREAM ? __builtin_nontemporal_load(p) : *p;
    const f32x4 v0 = f32x4{widen_bf16_lo(w.x), widen_bf16_hi(w.x), widen_bf16_lo(w.y), widen_bf16_hi(w.y)};
    const f32x4 v1 = f32x4{widen_bf16_lo(w.z), widen_bf16_hi(w.z), widen_bf16_lo(w.w), widen_bf16_hi(w.w)};
    const f32x4 r0 = standardise_quad<FAST>(v0, t);
    f32x4 r1;
    if constexpr (FSTATIC != 0) r1 = standardise_quad<FAST>(v1, t);
    else r1 = standardise_quad<FAST>(v1, quad_stats<0, FAST>(2 * oct + 1, a));
    u32x4 o;
    o.x = bf16_bits(r0.x) | (bf16_bits(r0.y) << 16);
    o.y = bf16_bits(r0.z) | (bf16_bits(r0.w) << 16);
    o.z = bf16_bits(r1.x) | (bf16_bits(r1.y) << 16);
    o.w = bf16_bits(r1.z) | (bf16_bits(r1.w) << 16);
    return o;
}

// Span kernel on octs: units_x / units_total count octs.
template <int FSTATIC, int THREADS, bool STREAM, bool FAST>
__global__ void __launch_bounds__(THREADS) gather_octs_kernel(GatherArgs a) {
    const uint32_t j = blockIdx.y;
    const uint32_t o = blockIdx.x * THREADS + threadIdx.x;
    const int64_t e0 = span_offset(a, j);
    const QuadStats t = quad_stats<FSTATIC, FAST>(2 * o, a);
    pin_uniform<FSTATIC>(t);
    if (o >= a.units_total) return;
    void* dst = quad_destination<false>(a, j, o);  // an oct of bf16 is 16 bytes, like a quad of fp32
    const u32x4 r = standardised_oct<FSTATIC, STREAM, FAST>(a.series, e0 + 8ll * o, o, t, a);
    stream_store_16<true>(dst, __builtin_bit_cast(f32x4, r));
}

// Row kernel on octs: row_quads counts octs per row.
template <int FSTATIC, int THREADS, bool STREAM, bool FAST>
__global__ void __launch_bounds__(THREADS) gather_rows_octs_kernel(RowArgs a) {
    const uint32_t run = blockIdx.z, rr = blockIdx.y;
    const uint32_t o = blockIdx.x * THREADS + threadIdx.x;
    const uint32_t first_sample = run * a.B;
    const uint32_t run_len = min(a.B, a.count - first_sample);
    int32_t s0 = a.g.starts[first_sample];
    const int32_t s0_max = a.g.last_start - static_cast<int32_t>(run_len - 1);
    s0 = s0 < 0 ? 0 : (s0 > s0_max ? s0_max : s0);
    const QuadStats t = quad_stats<FSTATIC, FAST>(2 * o, a.g);
    pin_uniform<FSTATIC>(t);
    if (rr >= run_len + a.PQ - 1 || o >= a.row_quads) return;
    const int64_t e = (static_cast<int64_t>(s0) + rr) * a.g.R + 8ll * o;
    const u32x4 r = standardised_oct<FSTATIC, STREAM, FAST>(a.g.series, e, o, t, a.g);
    const uint32_t j_lo = (rr >= a.PQ - 1) ? rr - (a.PQ - 1) : 0u;
    const uint32_t j_hi = (rr < run_len - 1) ? rr : run_len - 1;
    const uint32_t Q = a.PQ - a.P;
    for (uint32_t j = j_lo; j <= j_hi; ++j) {
        const uint32_t p = rr - j;
        const size_t sample = first_sample + j;
        u32x4* dst = (p < a.P) ? static_cast<u32x4*>(a.g.out_x) + (sample * a.P + p) * a.row_quads + o
                               : static_cast<u32x4*>(a.g.out_y) + (sample * Q + (p - a.P)) * a.row_quads + o;
        stream_store_16<true>(dst, __builtin_bit_cast(f32x4, r));
    }
}

// Any geometry (P*R or Q*R not a multiple of 4): one element per thread.
template <int STORE_BYTES, bool OUT_BF16>
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
    const bool in_x = e < a.units_x;
    const size_t at = in_x ? static_cast<size_t>(j) * a.units_x + e
                           : static_cast<size_t>(j) * (a.units_total - a.units_x) + (e - a.units_x);
    void* base = in_x ? a.out_x : a.out_y;
    if constexpr (OUT_BF16) static_cast<uint16_t*>(base)[at] = static_cast<uint16_t>(bf16_bits(r));
    else static_cast<float*>(base)[at] = r;
}

// Turns run-time switches into template arguments: fn receives std::true_type or std::false_type.
template <typename Fn>
void with_bool(bool v, Fn&& fn) {
    if (v) fn(std::true_type{});
    else fn(std::false_type{});
}

struct Switches {
    bool stream_loads, fast_divide, out_bf16;
};

template <int STORE_BYTES, int FSTATIC, int THREADS>
void launch_quads_t(const GatherArgs& a, int32_t count, Switches sw, hipStream_t s) {
    dim3 grid((a.units_total + THREADS - 1) / THREADS, count), block(THREADS);
    with_bool(sw.stream_loads, [&](auto st) {
        with_bool(sw.fast_divide, [&](auto fa) {
            with_bool(sw.out_bf16, [&](auto ob) {
                hipLaunchKernelGGL((gather_quads_kernel<STORE_BYTES, FSTATIC, THREADS, decltype(st)::value,
                                                        decltype(fa)::value, decltype(ob)::value>),
                                   grid, block, 0, s, a);
            });
        });
    });
}

template <int STORE_BYTES, int FSTATIC>
void launch_quads(const GatherArgs& a, int32_t count, Switches sw, hipStream_t s) {
    // 512-lane workgroups for long samples (fewer workgroups to dispatch), 256 otherwise.
    if (a.units_total >= 32768u) launch_quads_t<STORE_BYTES, FSTATIC, 512>(a, count, sw, s);
    else launch_quads_t<STORE_BYTES, FSTATIC, 256>(a, count, sw, s);
}

template <int STORE_BYTES, int FSTATIC>
void launch_rows(const RowArgs& a, Switches sw, hipStream_t s) {
    constexpr int kT = 256;
    const uint32_t runs = (a.count + a.B - 1) / a.B;
    dim3 grid((a.row_quads + kT - 1) / kT, a.B + a.PQ - 1, runs), block(kT);
    with_bool(sw.stream_loads, [&](auto st) {
        with_bool(sw.fast_divide, [&](auto fa) {
            with_bool(sw.out_bf16, [&](auto ob) {
                hipLaunchKernelGGL((gather_rows_kernel<STORE_BYTES, FSTATIC, kT, decltype(st)::value,
                                                       decltype(fa)::value, decltype(ob)::value>),
                                   grid, block, 0, s, a);
            });
        });
    });
}

template <int FSTATIC>
void launch_octs(const GatherArgs& a, int32_t count, Switches sw, hipStream_t s) {
    constexpr int kT = 256;
    dim3 grid((a.units_total + kT - 1) / kT, count), block(kT);
    with_bool(sw.stream_loads, [&](auto st) {
        with_bool(sw.fast_divide, [&](auto fa) {
            hipLaunchKernelGGL((gather_octs_kernel<FSTATIC, kT, decltype(st)::value, decltype(fa)::value>), grid, block,
                               0, s, a);
        });
    });
}

template <int FSTATIC>
void launch_rows_octs(const RowArgs& a, Switches sw, hipStream_t s) {
    constexpr int kT = 256;
    const uint32_t runs = (a.count + a.B - 1) / a.B;
    dim3 grid((a.row_quads + kT - 1) / kT, a.B + a.PQ - 1, runs), block(kT);
    with_bool(sw.stream_loads, [&](auto st) {
        with_bool(sw.fast_divide, [&](auto fa) {
            hipLaunchKernelGGL((gather_rows_octs_kernel<FSTATIC, kT, decltype(st)::value, decltype(fa)::value>), grid,
                               block, 0, s, a);
        });
    });
}

// Picks the feature pattern: 1, 2 and 4 features are compile-time patterns, anything else generic.
template <int STORE_BYTES, typename Fn>
void with_feature_pattern(uint32_t F, Fn&& fn) {
    if (F == 1) fn(std::integral_constant<int, 1>{});
    else if (F == 2) fn(std::integral_constant<int, 2>{});
    else if (F == 4) fn(std::integral_constant<int, 4>{});
    else fn(std::integral_constant<int, 0>{});
}

template <int STORE_BYTES>
void launch_for_storage(const pgti_ctx* c, GatherArgs& a, int32_t count, bool out_bf16, hipStream_t s) {
    const int64_t ex = static_cast<int64_t>(c->P) * c->R, et = static_cast<int64_t>(c->P + c->Q) * c->R;
    const bool big_series = c->series_bytes > (256ull << 20);
    if (c->share_consecutive && c->R % 4 == 0 && c->B + c->P + c->Q - 1 <= 65535 &&
        (count + c->B - 1) / c->B <= 65535) {
        // Batches of consecutive starts: fetch every source row once (d_starts is batch aligned).
        RowArgs ra{};
        ra.g = a;
        ra.B = static_cast<uint32_t>(c->B);
        ra.count = static_cast<uint32_t>(count);
        ra.P = static_cast<uint32_t>(c->P);
        ra.PQ = static_cast<uint32_t>(c->P + c->Q);
        ra.row_quads = static_cast<uint32_t>(c->R / 4);
        const Switches sw{big_series, c->fast_divide, out_bf16};
        if (STORE_BYTES == 2 && out_bf16 && c->R % 8 == 0) {
            ra.row_quads = static_cast<uint32_t>(c->R / 8);  // octs per row
            with_feature_pattern<STORE_BYTES>(a.F, [&](auto fs) { launch_rows_octs<decltype(fs)::value>(ra, sw, s); });
        } else {
            with_feature_pattern<STORE_BYTES>(a.F, [&](auto fs) { launch_rows<STORE_BYTES, decltype(fs)::value>(ra, sw, s); });
        }
    } else if (c->path == GatherPath::kQuads) {
        a.units_x = static_cast<uint32_t>(ex / 4);
        a.units_total = static_cast<uint32_t>(et / 4);
        // Non-temporal loads once the series cannot live in the 256 MB last-level cache anyway
        // (with consecutive starts the rows are re-read by neighbouring samples: keep them cached).
        const Switches sw{big_series && !c->share_consecutive, c->fast_divide, out_bf16};
        if (STORE_BYTES == 2 && out_bf16 && ex % 8 == 0 && et % 8 == 0) {
            a.units_x = static_cast<uint32_t>(ex / 8);  // octs
            a.units_total = static_cast<uint32_t>(et / 8);
            with_feature_pattern<STORE_BYTES>(a.F, [&](auto fs) { launch_octs<decltype(fs)::value>(a, count, sw, s); });
        } else {
            with_feature_pattern<STORE_BYTES>(a.F, [&](auto fs) { launch_quads<STORE_BYTES, decltype(fs)::value>(a, count, sw, s); });
        }
    } else {
        a.units_x = static_cast<uint32_t>(ex);
        a.units_total = static_cast<uint32_t>(et);
        dim3 grid((a.units_total + kThreads - 1) / kThreads, count);
        if (out_bf16) hipLaunchKernelGGL((gather_scalar_kernel<STORE_BYTES, true>), grid, dim3(kThreads), 0, s, a);
        else hipLaunchKernelGGL((gather_scalar_kernel<STORE_BYTES, false>), grid, dim3(kThreads), 0, s, a);
    }
}

}  // namespace

hipError_t launch_batch_gather(const pgti_ctx* c, const int32_t* d_starts, int32_t count, void* out_x, void* out_y,
                               bool out_bf16, hipStream_t s) {
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
        a.recip[f] = c->recip[f];
    }
    a.d_mean = c->d_stats;
    a.d_std = c->d_stats + c->F;
    a.d_recip = c->d_stats + 2 * c->F;
    if (c->storage == PGTI_F32) launch_for_storage<4>(c, a, count, out_bf16, s);
    else launch_for_storage<2>(c, a, count, out_bf16, s);
    return hipGetLastError();
}

}  // namespace pgti
