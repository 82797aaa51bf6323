// Internal declarations of the gfx950 index-batching library: the context behind the opaque
// handle of pgti.h and the kernel launchers each translation unit provides.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "pgti.h"

namespace pgti {

// Features whose statistics travel inside the kernel argument block; larger F reads them from HBM.
constexpr int kInlineStats = 8;
// Streams whose batch builds are tracked between two epoch-index generations.
constexpr int kMaxTrackedStreams = 8;

struct TrackedStream {
    hipStream_t stream;
    hipEvent_t event;  // recorded behind the builds of this stream when the next sort is enqueued
};

// How pgti_build_batch maps a sample onto threads, fixed when the series is loaded.
enum class GatherPath : int {
    kScalar = 0,  // any geometry: one element per thread
    kQuads = 1    // P*R and Q*R multiples of 4: one 16-byte output quad per thread-iteration
};

}  // namespace pgti

struct pgti_ctx {
    int device = 0;

    // geometry (valid when loaded)
    bool loaded = false;
    int64_t T = 0;
    int32_t N = 0, F = 0, P = 0, Q = 0, B = 0;
    pgti_dtype storage = PGTI_F32;
    int64_t R = 0;          // elements per timestep row, N*F
    int64_t n_windows = 0;  // T - (P+Q) + 1

    // resident store
    void* d_series = nullptr;
    size_t series_bytes = 0;
    std::vector<float> mean, stdev;  // host copies, F entries
    std::vector<float> recip;        // RN(1 / stdev[f]) for the gather's fast division
    bool fast_divide = false;        // every stdev[f] inside the range the fast division is valid for
    float* d_stats = nullptr;        // device: mean[F], std[F], recip[F]
    pgti::GatherPath path = pgti::GatherPath::kScalar;

    // epoch index generation
    hipStream_t work_stream = nullptr;  // owns the sort and the load-time kernels
    uint64_t* d_keys[2] = {nullptr, nullptr};
    int32_t* d_vals[2] = {nullptr, nullptr};
    uint32_t* d_hist = nullptr;                // per-(digit, tile) counts of the current pass (radix path)
    uint32_t* d_tot = nullptr;                 // [256] digit totals of the current pass (radix path)
    uint32_t* d_bucket = nullptr;              // bucket path: totals, cursors, offsets (see kSortBucketWords)
    uint32_t bucket_sort_cap = 0;              // largest bucket that is ordered in LDS
    uint64_t sort_key_mask = ~0ull;            // all ones; a test hook clears low bits to force equal keys
    int32_t* d_share = nullptr;                // this rank's starts, capacity n_windows (what the builds read)
    int32_t* d_share_next = nullptr;           // where the next order is computed while builds still read d_share
    uint32_t sort_blocks = 0;
    bool have_share = false;
    bool share_consecutive = false;  // batches hold consecutive starts (sequential / batch-shuffled order)
    int64_t share_lo = 0, share_hi = 0;
    hipEvent_t ev_share_ready = nullptr;

    pgti::TrackedStream tracked[pgti::kMaxTrackedStreams];
    int n_tracked = 0;
};

namespace pgti {

// ---- error plumbing (pgti_api.hip) ----------------------------------------------------------
int fail(int status, const char* fmt, ...);
int fail_hip(hipError_t e, const char* what);
void clear_error();

#define PGTI_HIP_TRY(expr)                                   \
    do {                                                     \
        hipError_t e__ = (expr);                             \
        if (e__ != hipSuccess) return ::pgti::fail_hip(e__, #expr); \
    } while (0)

// ---- series_store.hip -----------------------------------------------------------------------
// One streaming pass over a chunk of `rows` source rows (fp32, [rows][N * F_src], device):
//   * dst != nullptr: the resident rows [rows][N * F] are written, fp32 or bf16 (rounded to nearest
//     even).  F_src == F - 1 (with period > 0) appends the time-of-day feature (t mod period) /
//     period of the row to every node; otherwise F_src == F.
//   * row_acc != nullptr: row_acc[(row0 + r) * F + f] receives, in fp64, the sum over the nodes in
//     node order of the fp32 values of feature f of row r (mean64 == nullptr) or of their squared
//     deviations from mean64[f] (device).  row_acc is [rows of the whole series][F] on the device.
// row0 is the absolute index of the chunk's first row.
hipError_t launch_ingest_rows(const float* src, int64_t rows, int32_t N, int32_t F, int32_t F_src, int32_t period,
                              int64_t row0, void* dst, bool dst_bf16, const double* mean64, double* row_acc,
                              hipStream_t s);
// Algorithm 1's scalar statistic over the first n_train windows of x: weighted sum of the row sums
// over count = n_train*P*N*F elements, written to all F entries of out64 / out32.
hipError_t launch_reduce_rows_alg1(const double* row_acc, int32_t F, int64_t n_train, int32_t P, double count,
                                   bool take_sqrt, double* out64, float* out32, hipStream_t s);
// Adds the T row sums of every feature in time order, divides by T*N; take_sqrt selects the
// standard deviation.  out64 is [F] fp64 on the device, out32 [F] fp32 on the device.
hipError_t launch_reduce_rows(const double* row_acc, int64_t T, int32_t N, int32_t F, bool take_sqrt,
                              double* out64, float* out32, hipStream_t s);

// ---- epoch_sort.hip -------------------------------------------------------------------------
constexpr uint32_t kSortTile = 2048;          // keys per workgroup per pass
constexpr uint32_t kMaxSortBuckets = 1024;    // bucket path: buckets of the top key bits
constexpr uint32_t kBucketSortKeys = 2048;    // bucket path: largest bucket ordered in LDS
constexpr uint32_t kBucketPathKeys = 1u << 20;  // bucket path up to this many keys; beyond, the radix passes are as fast or faster
// d_bucket: tot[kMaxSortBuckets], cursor[kMaxSortBuckets], off[kMaxSortBuckets + 1]; tot and cursor
// must be zero when a sort starts (zeroed at allocation, and by the last kernel of every sort).
constexpr uint32_t kSortBucketWords = 3 * kMaxSortBuckets + 1;
// One sorted order: n_keys keys key(seed, epoch, counter_base + i*counter_stride) ordered by
// (key, i); positions [out_lo, out_hi) of the sorted index list, plus value_offset, land in out[].
// out may be c->d_vals[0] (free during the last pass) when the order is an intermediate result.
struct SortPlan {
    uint32_t n_keys;
    uint64_t counter_base, counter_stride;
    int32_t* out;
    uint32_t out_lo, out_hi;
    int32_t value_offset;
};
// Device memory a sort works in.  The bucket path (n_keys <= kBucketPathKeys) touches only keys[1],
// vals[1] and bucket; the single-workgroup path (n_keys <= 1,024) touches none of it.
struct SortWorkspace {
    uint64_t* keys[2];
    int32_t* vals[2];
    uint32_t* hist;           // per-(digit, tile) counts of the current pass (radix path)
    uint32_t* tot;            // [256] digit totals of the current pass (radix path)
    uint32_t* bucket;         // kSortBucketWords words (bucket path)
    uint32_t bucket_sort_cap; // largest bucket that is ordered in LDS
    uint64_t key_mask;        // ANDed onto every key: all ones, except under the test hook that forces ties
};
hipError_t launch_sorted_order(const SortWorkspace& w, uint64_t seed, uint64_t epoch, const SortPlan& plan,
                               hipStream_t s);
// The per-device address of the file-scope scratch array behind pgti_epoch_indices_static; resolves
// it on the first call for `device`, which must be the current device.  No allocation.
hipError_t static_sort_scratch(int device, void** ptr);
hipError_t launch_sequential_order(int32_t* share, uint32_t len, int32_t first, hipStream_t s);
hipError_t launch_expand_batches(const int32_t* order, uint32_t n_full, uint32_t B, int32_t base, int32_t* share,
                                 uint32_t len, hipStream_t s);

// ---- batch_gather.hip -----------------------------------------------------------------------
// Enqueues the fused gather + standardise of `count` samples whose starts are d_starts[0..count);
// outputs fp32, or bf16 (out_bf16) rounded to nearest even from the fp32 result.
hipError_t launch_batch_gather(const pgti_ctx* c, const int32_t* d_starts, int32_t count, void* out_x, void* out_y,
                               bool out_bf16, hipStream_t s);

}  // namespace pgti
