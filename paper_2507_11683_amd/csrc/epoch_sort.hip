// Epoch index generation (Sec. 4.2 of the paper: the dataset is shuffled at the start of each
// epoch and then partitioned according to the number of workers).
//
// The shuffle is defined as the order of the starts 0..n-1 under ascending (key_i, i), with
// key_i = M((h1 ^ i) + g), h1 = M((h0 ^ epoch) + g), h0 = M(seed + g), M the splitmix64 output
// function.
//
// Three ways to get that order, by the number of keys n:
//   n <= 1,024       one launch of one workgroup: keys are generated into LDS and ordered by
//                    (key, index) with a bitonic network.
//   n <= 1,048,576   (every benchmark workload) three launches: count the keys per bucket of the top
//                    4..10 key bits; scatter every (key, index) into its bucket (place inside the
//                    bucket arbitrary: LDS and global integer atomics); one workgroup per bucket
//                    orders its few hundred pairs in LDS, again by (key, index).  The pairs are all
//                    distinct, so the result does not depend on the order the atomics resolved in.
//   larger n         a least-significant-digit radix sort: 8 stable counting passes over 8-bit
//                    digits, the index riding along as the value (stability of every pass makes the
//                    index the tiebreak).  One pass = three launches:
//   count   : per-(digit, workgroup) counts of the pass's digit, from an LDS histogram per tile (the
//             key generation launch produces those of pass 0).  Counting the next pass's digit
//             during the scatter instead, one global atomic per key into the destination tile's
//             column, measured 6 times slower per pass (160 against 25 us at 4.5 M keys).
//   scan    : exclusive prefix over workgroups of the per-(digit, workgroup) counts, digit totals
//   scatter : each workgroup ranks its tile (wave ballots give every key its rank among equal
//             digits in its wave; per-wave LDS counters chain the rounds), puts the tile in digit
//             order in LDS, adds the scanned base and writes key/value to the destination in runs
//             of equal digits.
//
// Other orders reuse the same machinery: the sequential order (validation / test passes over a
// range of starts, Sec. 3.1) is an iota; the batch-level shuffle of Sec. 5.4 (fixed partition,
// batch order shuffled, batch contents fixed) sorts one key per full batch and expands the sorted
// batch numbers into starts.
#include <mutex>

#include "pgti_internal.h"

namespace pgti {
namespace {

constexpr uint32_t kThreads = 256;
constexpr uint32_t kWave = 64;
constexpr uint32_t kWaves = kThreads / kWave;
constexpr uint32_t kItems = kSortTile / kThreads;  // rounds per wave: 8
constexpr uint32_t kRadix = 256;
constexpr uint64_t kGamma = 0x9E3779B97F4A7C15ull;
static_assert(kRadix == kThreads, "one thread per digit in the scan steps");
static_assert(kItems * kThreads == kSortTile, "tile must be a whole number of rounds");

__device__ __forceinline__ uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Inclusive scan of one value per thread over the 256 threads of the workgroup.
__device__ __forceinline__ uint32_t block_inclusive_scan(uint32_t v, uint32_t* lds) {
    const uint32_t tid = threadIdx.x;
    lds[tid] = v;
    __syncthreads();
#pragma unroll
    for (uint32_t off = 1; off < kThreads; off <<= 1) {
        uint32_t t = (tid >= off) ? lds[tid - off] : 0u;
        __syncthreads();
        lds[tid] += t;
        __syncthreads();
    }
    uint32_t r = lds[tid];
    __syncthreads();
    return r;
}

// keys[i] = key(seed, epoch, counter_base + i*counter_stride) for i < n; counts of the lowest digit
// per (digit, workgroup) into hist0[digit][wg].
__global__ void __launch_bounds__(kThreads) keygen_kernel(uint64_t seed, uint64_t epoch, uint32_t n,
                                                          uint32_t nblk, uint64_t counter_base,
                                                          uint64_t counter_stride, uint64_t key_mask,
                                                          uint64_t* keys, uint32_t* hist0) {
    __shared__ uint32_t counts[kRadix];
    const uint32_t tid = threadIdx.x, b = blockIdx.x;
    counts[tid] = 0;
    __syncthreads();
    const uint64_t h0 = mix64(seed + kGamma);
    const uint64_t h1 = mix64((h0 ^ epoch) + kGamma);
#pragma unroll
    for (uint32_t it = 0; it < kItems; ++it) {
        uint32_t i = b * kSortTile + it * kThreads + tid;
        if (i < n) {
            uint64_t k = mix64((h1 ^ (counter_base + static_cast<uint64_t>(i) * counter_stride)) + kGamma) & key_mask;
            keys[i] = k;
            atomicAdd(&counts[k & 0xFFu], 1u);
        }
    }
    __syncthreads();
    hist0[tid * nblk + b] = counts[tid];
}

// counts of the digit at `shift` per (digit, workgroup) into hist[digit][wg], for the keys as they lie
// before the pass that sorts by that digit.
__global__ void __launch_bounds__(kThreads) digit_count_kernel(const uint64_t* __restrict__ keys, uint32_t n,
                                                               uint32_t nblk, uint32_t shift,
                                                               uint32_t* __restrict__ hist) {
    __shared__ uint32_t counts[kRadix];
    const uint32_t tid = threadIdx.x, b = blockIdx.x;
    counts[tid] = 0;
    __syncthreads();
#pragma unroll
    for (uint32_t it = 0; it < kItems; ++it) {
        const uint32_t i = b * kSortTile + it * kThreads + tid;
        if (i < n) atomicAdd(&counts[static_cast<uint32_t>(keys[i] >> shift) & 0xFFu], 1u);
    }
    __syncthreads();
    hist[tid * nblk + b] = counts[tid];
}

// One workgroup per digit d: hist[d][0..nblk) becomes its exclusive prefix, tot[d] its sum.
__global__ void __launch_bounds__(kThreads) scan_kernel(uint32_t* hist, uint32_t* tot, uint32_t nblk) {
    __shared__ uint32_t lds[kThreads];
    const uint32_t tid = threadIdx.x, d = blockIdx.x;
    uint32_t* row = hist + static_cast<size_t>(d) * nblk;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < nblk; base += kThreads) {
        uint32_t i = base + tid;
        uint32_t v = (i < nblk) ? row[i] : 0u;
        uint32_t incl = block_inclusive_scan(v, lds);
        if (i < nblk) row[i] = carry + incl - v;
        __shared__ uint32_t chunk_total;
        if (tid == kThreads - 1) chunk_total = incl;
        __syncthreads();
        carry += chunk_total;
        __syncthreads();
    }
    if (tid == 0) tot[d] = carry;
}

// Stable scatter of one tile by the digit at `shift`.
// FIRST: values are the element positions themselves (no value array yet).
// LAST : only the values whose destination falls in [lo, hi) are written, to share[pos - lo],
//        with value_offset added (the first start of the range the positions refer to).
template <bool FIRST, bool LAST>
__global__ void __launch_bounds__(kThreads) scatter_kernel(
    const uint64_t* __restrict__ keys_in, const int32_t* __restrict__ vals_in,
    uint64_t* __restrict__ keys_out, int32_t* __restrict__ vals_out,
    const uint32_t* __restrict__ hist_scanned, const uint32_t* __restrict__ tot, uint32_t n, uint32_t nblk,
    uint32_t shift, int32_t* __restrict__ share, uint32_t lo, uint32_t hi, int32_t value_offset) {
    __shared__ uint32_t wave_counts[kWaves][kRadix];  // running counts, later wave-exclusive offsets
    __shared__ uint32_t digit_base[kRadix];
    __shared__ uint32_t tile_first[kRadix];  // where the digit's run starts inside the digit-ordered tile
    __shared__ uint32_t scan_tmp[kThreads];
    __shared__ uint64_t sorted_key[kSortTile];
    __shared__ int32_t sorted_val[kSortTile];

    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), w = tid / kWave, b = blockIdx.x;
#pragma unroll
    for (uint32_t k = 0; k < kWaves; ++k) wave_counts[k][tid] = 0;
    __syncthreads();

    // Wave w owns the contiguous elements [first, first + 64*kItems) of the tile, taken in kItems
    // rounds of 64 consecutive elements: element order = (wave, round, lane) order.
    const uint32_t first = b * kSortTile + w * (kWave * kItems);
    uint64_t key[kItems];
    int32_t val[kItems];
    uint32_t rank[kItems];
#pragma unroll
    for (uint32_t r = 0; r < kItems; ++r) {
        uint32_t i = first + r * kWave + lane;
        bool valid = i < n;
        key[r] = valid ? keys_in[i] : 0ull;
        if constexpr (FIRST) val[r] = static_cast<int32_t>(i);
        else val[r] = valid ? vals_in[i] : 0;
    }

    const uint64_t lanes_below = (1ull << lane) - 1ull;
#pragma unroll
    for (uint32_t r = 0; r < kItems; ++r) {
        const bool valid = (first + r * kWave + lane) < n;
        const uint32_t d = static_cast<uint32_t>(key[r] >> shift) & 0xFFu;
        // peers: the valid lanes of this wave holding the same digit
        uint64_t peers = __ballot(valid);
#pragma unroll
        for (uint32_t bit = 0; bit < 8; ++bit) {
            const bool one = (d >> bit) & 1u;
            const uint64_t m = __ballot(one);
            peers &= one ? m : ~m;
        }
        const uint32_t below = __popcll(peers & lanes_below);
        const uint32_t count = __popcll(peers);
        uint32_t base = 0;
        if (valid) base = wave_counts[w][d];  // every peer reads the count before the leader bumps it
        __builtin_amdgcn_wave_barrier();
        if (valid && below == 0) wave_counts[w][d] = base + count;
        __builtin_amdgcn_wave_barrier();
        rank[r] = base + below;  // rank among equal digits within this wave's elements
    }
    __syncthreads();

    // thread tid = digit: wave-exclusive offsets, the digit's place inside the tile, and the global
    // base of (digit, this tile)
    {
        uint32_t run = 0;
#pragma unroll
        for (uint32_t k = 0; k < kWaves; ++k) {
            uint32_t cnt = wave_counts[k][tid];
            wave_counts[k][tid] = run;
            run += cnt;
        }
        const uint32_t t = tot[tid];
        const uint32_t before = hist_scanned[static_cast<size_t>(tid) * nblk + b];
        const uint32_t incl = block_inclusive_scan(t, scan_tmp);
        digit_base[tid] = (incl - t) + before;
        const uint32_t incl_tile = block_inclusive_scan(run, scan_tmp);
        tile_first[tid] = incl_tile - run;
    }
    __syncthreads();

    // The tile is put in digit order in LDS first (stable: rank order inside a digit is the element
    // order), so that consecutive lanes then write consecutive destinations: equal digits of a tile
    // go to one contiguous run, instead of 2,048 isolated 8-byte writes.
#pragma unroll
    for (uint32_t r = 0; r < kItems; ++r) {
        const bool valid = (first + r * kWave + lane) < n;
        if (!valid) continue;
        const uint32_t d = static_cast<uint32_t>(key[r] >> shift) & 0xFFu;
        const uint32_t local = tile_first[d] + wave_counts[w][d] + rank[r];
        if (local >= kSortTile) continue;  // cannot happen with consistent counts
        sorted_key[local] = key[r];
        sorted_val[local] = val[r];
    }
    __syncthreads();
    const uint32_t tile_n = (n - b * kSortTile < kSortTile) ? n - b * kSortTile : kSortTile;
    for (uint32_t i = tid; i < tile_n; i += kThreads) {
        const uint64_t k64 = sorted_key[i];
        const uint32_t d = static_cast<uint32_t>(k64 >> shift) & 0xFFu;
        const uint32_t pos = digit_base[d] + (i - tile_first[d]);
        if (pos >= n) continue;  // cannot happen with consistent counts; never write out of bounds
        if constexpr (!LAST) {
            keys_out[pos] = k64;
            vals_out[pos] = sorted_val[i];
        } else {
            if (pos >= lo && pos < hi) share[pos - lo] = sorted_val[i] + value_offset;
        }
    }
}

// One workgroup orders up to kSmallSortKeys keys in LDS.  Slots n..m-1 (m = n rounded up to a power
// of two) hold the largest key with their own slot number as index, which is above every real
// index, so they end up behind the n real entries.
constexpr uint32_t kSmallSortKeys = 1024;
constexpr uint32_t kSmallSortThreads = 512;

__global__ void __launch_bounds__(kSmallSortThreads) small_sort_kernel(uint64_t seed, uint64_t epoch, uint32_t n,
                                                                        uint32_t m, uint64_t counter_base,
                                                                        uint64_t counter_stride, uint64_t key_mask,
                                                                        int32_t* __restrict__ share, uint32_t lo,
                                                                        uint32_t hi, int32_t value_offset) {
    __shared__ uint64_t key[kSmallSortKeys];
    __shared__ uint32_t idx[kSmallSortKeys];
    const uint32_t tid = threadIdx.x;
    const uint64_t h0 = mix64(seed + kGamma);
    const uint64_t h1 = mix64((h0 ^ epoch) + kGamma);
    for (uint32_t i = tid; i < m; i += kSmallSortThreads) {
        key[i] = (i < n) ? (mix64((h1 ^ (counter_base + i * counter_stride)) + kGamma) & key_mask) : ~0ull;
        idx[i] = i;
    }
    __syncthreads();
    for (uint32_t size = 2; size <= m; size <<= 1) {
        for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
            for (uint32_t t = tid; t < (m >> 1); t += kSmallSortThreads) {
                const uint32_t a = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                const uint32_t b = a + stride;
                const uint64_t ka = key[a], kb = key[b];
                const uint32_t ia = idx[a], ib = idx[b];
                const bool a_after_b = (ka > kb) || (ka == kb && ia > ib);
                const bool ascending = (a & size) == 0;
                if (a_after_b == ascending) {
                    key[a] = kb; key[b] = ka;
                    idx[a] = ib; idx[b] = ia;
                }
            }
            __syncthreads();
        }
    }
    for (uint32_t i = tid; i < n; i += kSmallSortThreads)
        if (i >= lo && i < hi) share[i - lo] = static_cast<int32_t>(idx[i]) + value_offset;
}

// ---- bucket path: count, scatter, one workgroup per bucket --------------------------------------
// Bucket of a key = its top `dbits` bits, D = 2^dbits <= kMaxSortBuckets buckets.  tot[], cursor[] (D
// entries each) are zero between sorts: the last kernel clears what the first two filled.
constexpr uint32_t kBucketBins = kMaxSortBuckets / kThreads;  // bins per thread in the offset scan: 4
static_assert(kBucketBins * kThreads == kMaxSortBuckets, "whole bins per thread");

__device__ __forceinline__ uint64_t epoch_key(uint64_t h1, uint64_t counter, uint64_t key_mask) {
    return mix64((h1 ^ counter) + kGamma) & key_mask;
}

__global__ void __launch_bounds__(kThreads) bucket_count_kernel(uint64_t seed, uint64_t epoch, uint32_t n,
                                                                uint64_t counter_base, uint64_t counter_stride,
                                                                uint64_t key_mask, uint32_t dbits,
                                                                uint32_t* __restrict__ tot) {
    __shared__ uint32_t hist[kMaxSortBuckets];
    const uint32_t tid = threadIdx.x, D = 1u << dbits;
    for (uint32_t bin = tid; bin < D; bin += kThreads) hist[bin] = 0;
    __syncthreads();
    const uint64_t h1 = mix64((mix64(seed + kGamma) ^ epoch) + kGamma);
#pragma unroll
    for (uint32_t it = 0; it < kItems; ++it) {
        const uint32_t i = blockIdx.x * kSortTile + it * kThreads + tid;
        if (i < n) atomicAdd(&hist[epoch_key(h1, counter_base + i * counter_stride, key_mask) >> (64 - dbits)], 1u);
    }
    __syncthreads();
    for (uint32_t bin = tid; bin < D; bin += kThreads) {
        const uint32_t cnt = hist[bin];
        if (cnt) atomicAdd(&tot[bin], cnt);
    }
}

// Writes (key, index) of every element of the tile into its bucket: bucket b occupies
// [off[b], off[b+1]) of keys_out / vals_out, off = exclusive prefix of tot (recomputed by every
// workgroup; workgroup 0 also stores it, with off[D] = n, for the next kernel).
__global__ void __launch_bounds__(kThreads) bucket_scatter_kernel(uint64_t seed, uint64_t epoch, uint32_t n,
                                                                  uint64_t counter_base, uint64_t counter_stride,
                                                                  uint64_t key_mask, uint32_t dbits,
                                                                  const uint32_t* __restrict__ tot,
                                                                  uint32_t* __restrict__ cursor,
                                                                  uint32_t* __restrict__ off,
                                                                  uint64_t* __restrict__ keys_out,
                                                                  int32_t* __restrict__ vals_out) {
    __shared__ uint32_t hist[kMaxSortBuckets];  // count of this tile per bucket
    __shared__ uint32_t base[kMaxSortBuckets];  // where this tile's share of the bucket starts
    __shared__ uint32_t scan_tmp[kThreads];
    const uint32_t tid = threadIdx.x, D = 1u << dbits;
    for (uint32_t bin = tid; bin < D; bin += kThreads) hist[bin] = 0;
    __syncthreads();
    const uint64_t h1 = mix64((mix64(seed + kGamma) ^ epoch) + kGamma);
    uint64_t key[kItems];
    uint32_t rank[kItems];
#pragma unroll
    for (uint32_t it = 0; it < kItems; ++it) {
        const uint32_t i = blockIdx.x * kSortTile + it * kThreads + tid;
        key[it] = epoch_key(h1, counter_base + i * counter_stride, key_mask);
        rank[it] = (i < n) ? atomicAdd(&hist[key[it] >> (64 - dbits)], 1u) : 0u;
    }
    // offsets of the buckets: thread tid owns bins [4 tid, 4 tid + 4)
    uint32_t t[kBucketBins], sum = 0;
#pragma unroll
    for (uint32_t u = 0; u < kBucketBins; ++u) {
        const uint32_t bin = tid * kBucketBins + u;
        t[u] = (bin < D) ? tot[bin] : 0u;
        sum += t[u];
    }
    uint32_t run = block_inclusive_scan(sum, scan_tmp) - sum;  // the scan's barriers also complete hist[]
#pragma unroll
    for (uint32_t u = 0; u < kBucketBins; ++u) {
        const uint32_t bin = tid * kBucketBins + u;
        if (bin < D) {
            const uint32_t cnt = hist[bin];
            if (cnt) base[bin] = run + atomicAdd(&cursor[bin], cnt);
            if (blockIdx.x == 0) off[bin] = run;
        }
        run += t[u];
    }
    if (blockIdx.x == 0 && tid == 0) off[D] = n;
    __syncthreads();
#pragma unroll
    for (uint32_t it = 0; it < kItems; ++it) {
        const uint32_t i = blockIdx.x * kSortTile + it * kThreads + tid;
        if (i >= n) continue;
        const uint32_t pos = base[key[it] >> (64 - dbits)] + rank[it];
        if (pos >= n) continue;  // cannot happen with consistent counts; never write out of bounds
        keys_out[pos] = key[it];
        vals_out[pos] = static_cast<int32_t>(i);
    }
}

// Workgroup b orders bucket b by (key, index) and writes the indices whose final position falls in
// [lo, hi) to share[pos - lo], plus value_offset.  Up to `cap` <= kBucketSortKeys pairs the bucket is
// ordered in LDS with a bitonic network (padding: largest key with an index above every real one);
// a larger bucket takes the slow way, the rank of every pair counted against the whole bucket.
__global__ void __launch_bounds__(kThreads) bucket_sort_kernel(const uint64_t* __restrict__ keys,
                                                               const int32_t* __restrict__ vals,
                                                               const uint32_t* __restrict__ off,
                                                               uint32_t* __restrict__ tot,
                                                               uint32_t* __restrict__ cursor, uint32_t n,
                                                               uint32_t cap, int32_t* __restrict__ share, uint32_t lo,
                                                               uint32_t hi, int32_t value_offset) {
    __shared__ uint64_t key[kBucketSortKeys];
    __shared__ uint32_t idx[kBucketSortKeys];
    const uint32_t tid = threadIdx.x, b = blockIdx.x;
    const uint32_t end = min(off[b + 1], n), begin = min(off[b], end), m = end - begin;  // never past the arrays
    if (tid == 0) {
        tot[b] = 0;
        cursor[b] = 0;
    }
    if (m == 0) return;
    if (m <= cap) {
        uint32_t m2 = 2;
        while (m2 < m) m2 <<= 1;
        for (uint32_t i = tid; i < m2; i += kThreads) {
            key[i] = (i < m) ? keys[begin + i] : ~0ull;
            idx[i] = (i < m) ? static_cast<uint32_t>(vals[begin + i]) : 0xFFFFFFFFu;
        }
        __syncthreads();
        for (uint32_t size = 2; size <= m2; size <<= 1) {
            for (uint32_t stride = size >> 1; stride > 0; stride >>= 1) {
                for (uint32_t t = tid; t < (m2 >> 1); t += kThreads) {
                    const uint32_t a = ((t & ~(stride - 1)) << 1) | (t & (stride - 1));
                    const uint32_t c = a + stride;
                    const uint64_t ka = key[a], kc = key[c];
                    const uint32_t ia = idx[a], ic = idx[c];
                    const bool a_after_c = (ka > kc) || (ka == kc && ia > ic);
                    const bool ascending = (a & size) == 0;
                    if (a_after_c == ascending) {
                        key[a] = kc; key[c] = ka;
                        idx[a] = ic; idx[c] = ia;
                    }
                }
                __syncthreads();
            }
        }
        for (uint32_t i = tid; i < m; i += kThreads) {
            const uint32_t pos = begin + i;
            if (pos >= lo && pos < hi) share[pos - lo] = static_cast<int32_t>(idx[i]) + value_offset;
        }
    } else {
        for (uint32_t e = tid; e < m; e += kThreads) {
            const uint64_t k = keys[begin + e];
            const int32_t v = vals[begin + e];
            uint32_t below = 0;
            for (uint32_t f = 0; f < m; ++f) {
                const uint64_t k2 = keys[begin + f];
                below += (k2 < k) || (k2 == k && vals[begin + f] < v);
            }
            const uint32_t pos = begin + below;
            if (pos >= lo && pos < hi) share[pos - lo] = v + value_offset;
        }
    }
}

// share[i] = first + i (sequential order).
__global__ void __launch_bounds__(kThreads) iota_kernel(int32_t* __restrict__ share, uint32_t len, int32_t first) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < len) share[i] = first + static_cast<int32_t>(i);
}

// Batch-level shuffle: element i of the share belongs to visit slot i / B; full batches are visited
// in `order`, the short remainder (slots >= n_full) stays in place.
__global__ void __launch_bounds__(kThreads) expand_batches_kernel(const int32_t* __restrict__ order,
                                                                  uint32_t n_full, uint32_t B, int32_t base,
                                                                  int32_t* __restrict__ share, uint32_t len) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i >= len) return;
    const uint32_t slot = i / B, j = i - slot * B;
    const uint32_t batch = (slot < n_full) ? static_cast<uint32_t>(order[slot]) : slot;
    share[i] = base + static_cast<int32_t>(batch * B + j);
}

}  // namespace

namespace {

void launch_pass(const SortWorkspace* c, uint32_t pass, uint32_t n, uint32_t nblk, const SortPlan& plan, hipStream_t s) {
    const uint64_t* kin = c->keys[pass & 1];
    const int32_t* vin = c->vals[pass & 1];
    uint64_t* kout = c->keys[(pass + 1) & 1];
    int32_t* vout = c->vals[(pass + 1) & 1];
    const dim3 grid(nblk), block(kThreads);
    if (pass == 0)
        hipLaunchKernelGGL((scatter_kernel<true, false>), grid, block, 0, s, kin, vin, kout, vout, c->hist, c->tot, n,
                           nblk, 8 * pass, plan.out, plan.out_lo, plan.out_hi, plan.value_offset);
    else if (pass < 7)
        hipLaunchKernelGGL((scatter_kernel<false, false>), grid, block, 0, s, kin, vin, kout, vout, c->hist, c->tot, n,
                           nblk, 8 * pass, plan.out, plan.out_lo, plan.out_hi, plan.value_offset);
    else
        hipLaunchKernelGGL((scatter_kernel<false, true>), grid, block, 0, s, kin, vin, kout, vout, c->hist, c->tot, n,
                           nblk, 8 * pass, plan.out, plan.out_lo, plan.out_hi, plan.value_offset);
}

}  // namespace

hipError_t launch_sorted_order(const SortWorkspace& w, uint64_t seed, uint64_t epoch, const SortPlan& plan,
                               hipStream_t s) {
    const SortWorkspace* c = &w;
    const uint32_t n = plan.n_keys;
    if (n == 0) return hipSuccess;
    if (n <= kSmallSortKeys) {
        uint32_t m = 1;
        while (m < n) m <<= 1;
        hipLaunchKernelGGL(small_sort_kernel, dim3(1), dim3(kSmallSortThreads), 0, s, seed, epoch, n, m,
                           plan.counter_base, plan.counter_stride, c->key_mask, plan.out, plan.out_lo, plan.out_hi,
                           plan.value_offset);
        return hipGetLastError();
    }
    const uint32_t nblk = (n + kSortTile - 1) / kSortTile;
    if (n <= kBucketPathKeys) {
        // buckets of a few hundred keys: the fewest top bits that bring the average to 384 or less
        uint32_t dbits = 4;
        while ((1u << dbits) < kMaxSortBuckets && (n >> dbits) > 384u) ++dbits;
        const uint32_t D = 1u << dbits;
        uint32_t* tot = c->bucket;
        uint32_t* cursor = c->bucket + kMaxSortBuckets;
        uint32_t* off = c->bucket + 2 * kMaxSortBuckets;
        hipLaunchKernelGGL(bucket_count_kernel, dim3(nblk), dim3(kThreads), 0, s, seed, epoch, n, plan.counter_base,
                           plan.counter_stride, c->key_mask, dbits, tot);
        hipLaunchKernelGGL(bucket_scatter_kernel, dim3(nblk), dim3(kThreads), 0, s, seed, epoch, n, plan.counter_base,
                           plan.counter_stride, c->key_mask, dbits, tot, cursor, off, c->keys[1], c->vals[1]);
        hipLaunchKernelGGL(bucket_sort_kernel, dim3(D), dim3(kThreads), 0, s, c->keys[1], c->vals[1], off, tot,
                           cursor, n, c->bucket_sort_cap, plan.out, plan.out_lo, plan.out_hi, plan.value_offset);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(keygen_kernel, dim3(nblk), dim3(kThreads), 0, s, seed, epoch, n, nblk, plan.counter_base,
                       plan.counter_stride, c->key_mask, c->keys[0], c->hist);
    for (uint32_t pass = 0; pass < 8; ++pass) {
        if (pass > 0)
            hipLaunchKernelGGL(digit_count_kernel, dim3(nblk), dim3(kThreads), 0, s, c->keys[pass & 1], n, nblk, 8 * pass,
                               c->hist);
        hipLaunchKernelGGL(scan_kernel, dim3(kRadix), dim3(kThreads), 0, s, c->hist, c->tot, nblk);
        launch_pass(c, pass, n, nblk, plan, s);
    }
    return hipGetLastError();
}

hipError_t launch_sequential_order(int32_t* share, uint32_t len, int32_t first, hipStream_t s) {
    if (len == 0) return hipSuccess;
    hipLaunchKernelGGL(iota_kernel, dim3((len + kThreads - 1) / kThreads), dim3(kThreads), 0, s, share, len, first);
    return hipGetLastError();
}

hipError_t launch_expand_batches(const int32_t* order, uint32_t n_full, uint32_t B, int32_t base, int32_t* share,
                                 uint32_t len, hipStream_t s) {
    if (len == 0) return hipSuccess;
    hipLaunchKernelGGL(expand_batches_kernel, dim3((len + kThreads - 1) / kThreads), dim3(kThreads), 0, s, order,
                       n_full, B, base, share, len);
    return hipGetLastError();
}

}  // namespace pgti

// ---- the epoch order for callers that cannot allocate ---------------------------------------------
// pgti_epoch_indices_static works in this file-scope array instead of a workspace from hipMalloc:
// bucketed keys u64[kStaticSortKeys], bucketed indices i32[kStaticSortKeys], then the bucket totals,
// cursors and offsets (kSortBucketWords words).  Every GPU the library runs on holds its own copy at
// its own address until the process ends; the name below is only a host-side handle for
// hipGetSymbolAddress, the kernels receive the resolved device pointer.
namespace pgti {
namespace {

constexpr uint32_t kStaticSortKeys = 1u << 20;  // 1,048,576 keys: the whole bucket path, ten times the paper's largest dataset
static_assert(kStaticSortKeys <= kBucketPathKeys, "the allocation-free call only has a workspace for the bucket path");
constexpr size_t kStaticKeysBytes = sizeof(uint64_t) * kStaticSortKeys;
constexpr size_t kStaticValsBytes = sizeof(int32_t) * kStaticSortKeys;
constexpr size_t kStaticBucketBytes = sizeof(uint32_t) * kSortBucketWords;
constexpr size_t kStaticScratchBytes = kStaticKeysBytes + kStaticValsBytes + ((kStaticBucketBytes + 255) / 256) * 256;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Zeroes `words` 32-bit words (a kernel, not a memset node, so that a caller may capture the call
// into a HIP graph).
__global__ void __launch_bounds__(kThreads) zero_words_kernel(uint32_t* __restrict__ p, uint32_t words) {
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < words) p[i] = 0u;
}

}  // namespace

hipError_t static_sort_scratch(int device, void** ptr) {
    *ptr = nullptr;
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // of the current device
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        g_scratch_ptr[device] = p;
    }
    *ptr = g_scratch_ptr[device];
    return hipSuccess;
}

}  // namespace pgti

extern "C" int64_t pgti_epoch_indices_static(int device, int64_t n_windows, uint64_t seed, uint64_t epoch,
                                              uint32_t rank, uint32_t world, int32_t* share_out, int64_t capacity,
                                              void* stream) {
    using namespace pgti;
    clear_error();
    if (n_windows <= 0) return fail(PGTI_ERR_ARG, "n_windows must be positive (got %lld)", (long long)n_windows);
    if (n_windows > static_cast<int64_t>(kStaticSortKeys))
        return fail(PGTI_ERR_RANGE, "%lld windows exceed the %u this allocation-free call is built for",
                    (long long)n_windows, kStaticSortKeys);
    if (world == 0) return fail(PGTI_ERR_RANGE, "world must be at least 1");
    if (rank >= world) return fail(PGTI_ERR_RANGE, "rank %u not in [0, %u)", rank, world);
    const uint64_t n = static_cast<uint64_t>(n_windows);
    const uint64_t lo = (static_cast<uint64_t>(rank) * n) / world, hi = ((static_cast<uint64_t>(rank) + 1) * n) / world;
    const int64_t len = static_cast<int64_t>(hi - lo);
    if (len > 0 && !share_out) return fail(PGTI_ERR_ARG, "null output pointer");
    if (capacity < len)
        return fail(PGTI_ERR_ARG, "share of %lld starts does not fit capacity %lld", (long long)len, (long long)capacity);
    if (reinterpret_cast<uintptr_t>(share_out) & 3u) return fail(PGTI_ERR_ARG, "share_out must be 4-byte aligned");
    if (len == 0) return 0;

    int prev = -1;
    PGTI_HIP_TRY(hipGetDevice(&prev));
    if (prev != device) PGTI_HIP_TRY(hipSetDevice(device));
    struct Restore {
        int prev, device;
        ~Restore() {
            if (prev != device) (void)hipSetDevice(prev);
        }
    } restore{prev, device};

    void* base = nullptr;
    PGTI_HIP_TRY(static_sort_scratch(device, &base));
    unsigned char* p = static_cast<unsigned char*>(base);
    SortWorkspace w{};
    w.keys[1] = reinterpret_cast<uint64_t*>(p);
    w.vals[1] = reinterpret_cast<int32_t*>(p + kStaticKeysBytes);
    w.bucket = reinterpret_cast<uint32_t*>(p + kStaticKeysBytes + kStaticValsBytes);
    w.bucket_sort_cap = kBucketSortKeys;
    w.key_mask = ~0ull;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // The array keeps whatever the last call left (also a call that was cut short): totals and
    // cursors must start at zero.
    if (n > kSmallSortKeys)
        hipLaunchKernelGGL(zero_words_kernel, dim3((2 * kMaxSortBuckets + kThreads - 1) / kThreads), dim3(kThreads), 0,
                           s, w.bucket, 2 * kMaxSortBuckets);
    const SortPlan plan{static_cast<uint32_t>(n), 0, 1, share_out, static_cast<uint32_t>(lo),
                        static_cast<uint32_t>(hi), 0};
    PGTI_HIP_TRY(launch_sorted_order(w, seed, epoch, plan, s));
    return len;
}
