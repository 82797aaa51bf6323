/*
 * pgti.h -- C ABI of the MI355X (gfx950) index-batching library.
 *
 * What it does (PGT-I, arXiv 2507.11683): instead of materialising every sliding-window
 * snapshot of a spatiotemporal series (Algorithm 1; size given by Eq. 1) and copying batches
 * host-to-device, ONE copy of the [T, N, F] series stays resident in HBM together with one
 * start index per window (Eq. 2), and each training batch is rebuilt on the device from start
 * indices (Sec. 4.1, "Index-Batching" and "GPU-Index-Batching").  Each epoch the starts are
 * shuffled and split by worker (Sec. 4.2).
 *
 * Conventions
 *   - Plain C linkage.  No exceptions or aborts cross the boundary.
 *   - Every function that returns int returns >= 0 on success and a negative pgti_status on
 *     failure; pgti_last_error() then describes it (thread-local string).
 *   - "host" / "device" in a comment says where a pointer must live.
 *   - The library owns the resident series, the statistics and the index buffers; the caller
 *     owns every pointer it passes in (host inputs may be freed as soon as the call returns)
 *     and the HIP stream.
 *   - A context is bound to one GPU and is not thread-safe.  Contexts are independent.
 *   - Layouts are row-major with the last index fastest: series [T, N, F];
 *     x [B, P, N, F]; y [B, Q, N, F].
 */
#ifndef PGTI_H
#define PGTI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct pgti_ctx pgti_ctx; /* opaque */

typedef enum {
    PGTI_F32 = 0, /* series stored as IEEE binary32 */
    PGTI_BF16 = 1 /* series stored as bfloat16 (fp32 rounded to nearest, ties to even) */
} pgti_dtype;

typedef enum {
    PGTI_OK = 0,
    PGTI_ERR_ARG = -1,   /* null pointer, non-positive size, misaligned output, bad enum */
    PGTI_ERR_STATE = -2, /* call order: no series loaded / no epoch indices generated */
    PGTI_ERR_RANGE = -3, /* batch_no beyond the share, rank >= world, T < P + Q, too many windows */
    PGTI_ERR_STATS = -4, /* a standard deviation is zero or a statistic is not finite */
    PGTI_ERR_OOM = -5,   /* device or pinned-host allocation failed */
    PGTI_ERR_HIP = -6    /* any other HIP runtime error (text in pgti_last_error) */
} pgti_status;

/* Creates a context on GPU `device` (ordinal as seen by HIP).  *out receives the handle. */
int pgti_create(pgti_ctx** out, int device);

/* Test hook for the epoch sort of this context (no effect on any other state; not for production).
 * bucket_cap: 0 = default; 1..2047 lowers the size up to which a bucket of keys is ordered in
 *     on-chip memory, so that the slow ordering path for oversized buckets runs; results do not
 *     depend on it.
 * key_bits: 0 or 64 = the full 64-bit keys (the distinct keys of Sec. 4.2's shuffle as defined at
 *     pgti_epoch_indices); 1..63 keeps only the top key_bits bits of every key, so that many starts
 *     share a key and the order among them is decided by the index alone (lower start first).
 *     This changes the epoch order: it exists to exercise the tie-break, which full keys never do.
 * Returns PGTI_OK or PGTI_ERR_ARG.  Takes effect at the next index generation. */
int pgti_set_sort_test_hooks(pgti_ctx* c, uint32_t bucket_cap, uint32_t key_bits);

/* Frees everything the context owns after waiting for the device work it enqueued on its own
 * stream and for the streams that received batch builds since the last epoch-index generation.
 * Streams must still exist at this point.  NULL is ok. */
void pgti_destroy(pgti_ctx* c);

/*
 * Resident store (Sec. 4.1, GPU-Index-Batching: the data is moved to GPU memory once; index
 * batching keeps a single copy of it, Eq. 2).
 *
 * Copies host_series (HOST, fp32, [T, N, F]) to HBM in `storage` precision and fixes the window
 * geometry: P input steps, Q target steps (the paper's single `horizon` is P = Q), batch size B.
 * The number of valid starts becomes n = T - (P + Q) + 1 (Eq. 1, Eq. 2).
 * mean, std: HOST, F floats each: the per-feature statistics used by pgti_build_batch
 * (Algorithm 1 standardises with (v - mu) / sigma).  If BOTH are NULL the library computes, on
 * the device, the mean and the population standard deviation of every feature over all T*N
 * values of the fp32 input.  Exactly one of them NULL is PGTI_ERR_ARG.
 * Replaces any series loaded before (after waiting for batch builds still in flight on it) and
 * invalidates its epoch indices -- but only when the load succeeds: the new store is built beside
 * the old one and swapped in at the end, so on ANY error the context keeps its previous series,
 * statistics and share and stays usable.  During the call both series occupy device memory; to
 * replace a series whose successor does not fit beside it, destroy the context and create a new one.
 * Synchronous: on return the host buffers are no longer referenced.
 * Errors: ARG, RANGE (T < P + Q, or n >= 2^31), STATS, OOM, HIP.
 */
int pgti_load_series(pgti_ctx* c, const float* host_series, int64_t T, int32_t N, int32_t F,
                     int32_t P, int32_t Q, int32_t B, pgti_dtype storage, const float* mean,
                     const float* std);

/* Same as pgti_load_series but the fp32 source already lives in DEVICE memory (for a caller
 * that produced or staged the series on the GPU).  The source is not modified or retained.
 * Ordering: the library reads the source on a stream of its own, so before the first read it waits
 * (hipDeviceSynchronize) for all work enqueued on the device so far, whatever stream produced the
 * series; work that writes the source must have been enqueued before this call.  The same holds
 * for pgti_load_series_ex with source_on_device != 0. */
int pgti_load_series_device(pgti_ctx* c, const float* device_series, int64_t T, int32_t N,
                            int32_t F, int32_t P, int32_t Q, int32_t B, pgti_dtype storage,
                            const float* mean, const float* std);

/*
 * Load with on-device preprocessing (Sec. 4.1: GPU-index-batching performs the preprocessing on the
 * GPU as well; Algorithm 1 and the data-growth figure of Sec. 3.3 name its steps).
 *
 * series: fp32 [T, N, F_in], HOST or (source_on_device != 0) DEVICE.
 * time_of_day_period > 0: stage 1 of the preprocessing, one more feature is appended to every
 *     node, (t mod period) / period (quotient in binary32), so the resident series has
 *     F = F_in + 1 features; 0: F = F_in.
 * stats_rule
 *     PGTI_STATS_GIVEN           mean / std (HOST, F entries each) as passed
 *     PGTI_STATS_FEATURE_GLOBAL  per feature: mean and population standard deviation of all T*N values
 *     PGTI_STATS_ALG1_TRAIN      Algorithm 1: ONE scalar mean and population standard deviation over
 *                                every element of x_train, the first round(train_fraction * n) windows
 *                                of the stacked x (round half to even; the listing uses 0.70); rows
 *                                near the ends of the training range count in fewer windows, features
 *                                are mixed; the scalar is used for every feature.
 *     Computed statistics are accumulated in fp64 on the device and rounded to fp32 once; they see
 *     the fp32 values (before any bf16 rounding), including the time-of-day feature.
 *     PGTI_STATS_FEATURE_GLOBAL fixes the order of the additions, so its result is reproducible to
 *     the bit on any machine: for each feature, every timestep row is summed node by node, the row
 *     sums are added in time order, mean = sum / (T*N); the squared deviations (v - mean)*(v - mean),
 *     difference and product each rounded to fp64, are summed the same way, std = sqrt(sum / (T*N)).
 *     PGTI_STATS_ALG1_TRAIN is evaluated as the window-count-weighted sum of the same row sums; it
 *     agrees with a literal window-by-window fp64 loop to within one fp32 unit in the last place.
 * Other fields as the arguments of pgti_load_series.  Errors: as pgti_load_series.
 */
typedef enum {
    PGTI_STATS_GIVEN = 0,
    PGTI_STATS_FEATURE_GLOBAL = 1,
    PGTI_STATS_ALG1_TRAIN = 2
} pgti_stats_rule;

typedef struct pgti_load_spec {
    int64_t T;
    int32_t N;
    int32_t F_in;               /* features in the source array */
    int32_t P, Q, B;
    int32_t storage;            /* a pgti_dtype */
    int32_t source_on_device;   /* 0: host pointer, 1: device pointer */
    int32_t stats_rule;         /* a pgti_stats_rule */
    int32_t time_of_day_period; /* 0: none */
    int32_t reserved;           /* set to 0 */
    double train_fraction;      /* PGTI_STATS_ALG1_TRAIN only */
    const float* mean;          /* PGTI_STATS_GIVEN only */
    const float* std;
} pgti_load_spec;

int pgti_load_series_ex(pgti_ctx* c, const float* series, const pgti_load_spec* spec);

/* Reads back the statistics in use (HOST, F floats each; either may be NULL). */
int pgti_get_stats(pgti_ctx* c, float* mean_out, float* std_out);

/*
 * Epoch index generation (Sec. 4.2: the dataset is shuffled at the start of each epoch, then
 * partitioned according to the number of workers; every worker holds the full data, so the
 * shuffle is global and needs no communication).
 *
 * The epoch order is the list of starts 0..n-1 sorted ascending by (key_i, i), where
 * key_i = M((h1 ^ i) + g), h1 = M((h0 ^ epoch) + g), h0 = M(seed + g), M the splitmix64 output
 * function and g = 0x9E3779B97F4A7C15; computed on the device (the pairs are all distinct, so
 * the order is unique whatever sorting method produces it).  Rank `rank` of `world` owns order[lo, hi), lo = floor(rank*n/world),
 * hi = floor((rank+1)*n/world): no padding, no dropping.  *n_share (HOST, may be NULL)
 * receives hi - lo.  Same arguments give the same bits on every run.
 * Replaces the previous share.  Stream ordering is handled inside: the new order is computed in a
 * staging buffer, concurrently with batch builds already enqueued through this context; a short
 * copy that publishes it waits for those builds, and later batch builds wait for that copy.
 * Does not block the host.
 * Errors: STATE (no series), RANGE (rank >= world, world == 0), HIP.
 */
int pgti_epoch_indices(pgti_ctx* c, uint64_t seed, uint64_t epoch, uint32_t rank, uint32_t world,
                       int64_t* n_share);

/*
 * Epoch index generation with an order and a range of starts.
 *
 * Range (Sec. 3.1: the windows are split 70/10/20 into train, validation and test; Algorithm 1
 * takes the training part as the leading windows): the epoch runs over the starts
 * [first_start, first_start + n_starts); n_starts < 0 means "to the last window".  Positions
 * inside the range are 0..n_starts-1 and rank `rank` of `world` owns the positions
 * [lo, hi) = [floor(rank*n_starts/world), floor((rank+1)*n_starts/world)) of the chosen order.
 *
 * order
 *   PGTI_ORDER_SHUFFLE        Sec. 4.2 global shuffle: positions sorted by (key(seed, epoch,
 *                             position), position); what pgti_epoch_indices does over all windows.
 *   PGTI_ORDER_SEQUENTIAL     time order (validation and test passes): the share is
 *                             first_start+lo .. first_start+hi-1.  seed and epoch are ignored.
 *   PGTI_ORDER_BATCH_SHUFFLE  Sec. 5.4: a fixed partition per worker, the order of the batches is
 *                             shuffled while the data inside a batch stays fixed.  The partition is
 *                             the sequential share [lo, hi), every epoch; it is cut into consecutive
 *                             batches of B positions; full batches are visited by ascending
 *                             (key(seed, epoch, position of the batch's first element), batch
 *                             number); a short remainder batch stays last.
 * A batch of B consecutive starts reads only B+P+Q-1 distinct rows for B*(P+Q) written ones.
 * Errors: ARG (null, unknown order), STATE, RANGE (rank/world, range outside the windows), HIP.
 */
typedef enum {
    PGTI_ORDER_SHUFFLE = 0,
    PGTI_ORDER_SEQUENTIAL = 1,
    PGTI_ORDER_BATCH_SHUFFLE = 2
} pgti_order;

typedef struct pgti_epoch_spec {
    int32_t order;       /* a pgti_order */
    int32_t reserved;    /* set to 0 */
    int64_t first_start; /* first start of the range */
    int64_t n_starts;    /* number of starts in the range; negative = all remaining windows */
    uint64_t seed;
    uint64_t epoch;
    uint32_t rank;
    uint32_t world;
} pgti_epoch_spec;

int pgti_epoch_indices_ex(pgti_ctx* c, const pgti_epoch_spec* spec, int64_t* n_share);

/*
 * Epoch index generation for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  (pgti_epoch_indices works in a
 * workspace that pgti_load_series allocated and needs a context; this call needs neither.)
 *
 * Same order, same split and same bits as pgti_epoch_indices for a series with `n_windows` valid
 * starts: the starts 0..n_windows-1 sorted by (key(seed, epoch, i), i), of which rank `rank` of
 * `world` owns order[lo, hi).  The share is written to share_out (DEVICE, int32, caller-owned,
 * room for `capacity` >= hi - lo entries) by kernels enqueued on `stream` (a hipStream_t as void*,
 * NULL = the default stream) of GPU `device`; the call returns without synchronising.
 * The sort works in a fixed array of 12.6 MB that is part of the library's device image (each GPU
 * the library runs on holds one copy until the process ends); its address is resolved once per
 * device, by pgti_create on that device or else by the first call.  The call makes no hipMalloc,
 * hipFree or other allocating call.
 * Limit: n_windows <= 1,048,576 (PGTI_STATIC_MAX_WINDOWS); more is PGTI_ERR_RANGE.
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different
 * streams, or threads) race and give undefined shares; calls on one stream are ordered and safe.
 * Returns hi - lo, or a negative pgti_status: ARG (n_windows <= 0, null or misaligned share_out,
 * capacity too small), RANGE (limit, rank >= world, world == 0), HIP.
 */
#define PGTI_STATIC_MAX_WINDOWS 1048576
int64_t pgti_epoch_indices_static(int device, int64_t n_windows, uint64_t seed, uint64_t epoch,
                                  uint32_t rank, uint32_t world, int32_t* share_out, int64_t capacity,
                                  void* stream);

/* Test hook: copies the current share to host_out (HOST, int32, room for `capacity` entries).
 * Blocks until the sort has finished.  Returns the share length, or ERR_ARG if it does not fit. */
int64_t pgti_get_indices(pgti_ctx* c, int32_t* host_out, int64_t capacity);

/* Number of batches in the current share, ceil(n_share / B); STATE if there is none. */
int64_t pgti_num_batches(pgti_ctx* c);

/*
 * Batch build = fused gather + standardise (Sec. 4.1: x = data[start : start+horizon],
 * y = data[start+horizon : start+2*horizon], rebuilt at run time from the start index;
 * Algorithm 1: (v - mu) / sigma).
 *
 * Batch `batch_no` holds the samples share[batch_no*B ... min((batch_no+1)*B, n_share)) in that
 * order.  For sample j with start s:  out_x[j, p, :, f] = (S[s+p, :, f] - mean[f]) / std[f],
 * p < P;  out_y[j, q, :, f] = (S[s+P+q, :, f] - mean[f]) / std[f], q < Q.  Every output has the
 * bits of two separately rounded IEEE binary32 operations, a subtraction and a correctly rounded
 * division (however the kernel arrives at that quotient); bf16 storage is widened exactly first.
 * out_x: DEVICE fp32 [B, P, N, F]; out_y: DEVICE fp32 [B, Q, N, F]; caller-owned, 16-byte
 * aligned.  `stream` is a hipStream_t passed as void* (NULL = the default stream).  The kernel
 * is enqueued and the call returns without synchronising.  The stream must stay alive until the
 * next epoch-index generation, load or destroy call on this context has returned: those calls
 * order themselves behind the builds enqueued on it.  The first build on a stream after an index
 * generation also makes that stream wait for the share (an event wait); every further build on it
 * is kernel launches only and may be recorded into a HIP graph by stream capture.  Such a graph
 * stays valid for later epochs of the same share length (its arguments do not change); replay it
 * behind one ordinary build on the same stream, which supplies the wait.
 * Streams: the context tracks up to 8 distinct streams between two index generations without
 * blocking; a build on a ninth distinct stream first waits ON THE HOST (hipStreamSynchronize) for
 * the oldest tracked stream and takes its slot.
 * Throughput: consecutive launches on ONE stream are dependent, and on MI355X the drain of one
 * launch plus the ramp of the next costs about 2.4 us per launch (a 23 us Statewide batch: 73 % of
 * the HBM peak).  Batches are independent, so a caller that wants one call per batch should
 * alternate its calls over TWO streams (batch b on stream b mod 2; 79 % measured), provided the two
 * streams sit on different hardware queues (HIP deals streams onto a few queues in creation
 * order); or build several batches per launch with pgti_build_batches.
 * Returns the number of valid samples B' in 1..B.  A short last batch is not padded: rows
 * j >= B' of the outputs are left untouched.
 * Errors: STATE, RANGE (batch_no outside [0, num_batches)), ARG (null or misaligned), HIP.
 */
int pgti_build_batch(pgti_ctx* c, int64_t batch_no, float* out_x, float* out_y, void* stream);

/*
 * Several batches per launch (Sec. 4.1: batches are generated on demand from a set of indices;
 * nothing ties one launch to one batch).  Builds the `k` consecutive batches
 * first_batch .. first_batch+k-1 of the current share with one kernel launch (per 65,535 samples), which removes the
 * launch-to-launch gaps that dominate small batches and cost about 2.4 us per launch on MI355X.
 * Same arithmetic and layout as pgti_build_batch: batch first_batch+i occupies slot i of
 * out_x: DEVICE fp32 [k, B, P, N, F] and out_y: DEVICE fp32 [k, B, Q, N, F] (caller-owned, 16-byte
 * aligned).  Only the last batch of the share can be short; it is not padded and the rows after its
 * B' samples are left untouched.  first_batch + k may not exceed pgti_num_batches().
 * Returns the total number of valid samples written, or a negative pgti_status
 * (STATE, RANGE, ARG, HIP as for pgti_build_batch).  Does not synchronise.
 */
int64_t pgti_build_batches(pgti_ctx* c, int64_t first_batch, int32_t k, float* out_x, float* out_y,
                           void* stream);

/*
 * Reduced-precision outputs (not in the paper; halves the bytes written per batch).  Same as
 * pgti_build_batches, but every standardised fp32 value (Algorithm 1: (v - mu) / sigma, computed
 * exactly as for the fp32 outputs) is rounded to bfloat16, nearest even, as the last step.
 * out_x: DEVICE bf16 [k, B, P, N, F], out_y: DEVICE bf16 [k, B, Q, N, F] as 16-bit patterns,
 * caller-owned, 16-byte aligned.  Returns the number of valid samples or a negative pgti_status.
 */
int64_t pgti_build_batches_bf16(pgti_ctx* c, int64_t first_batch, int32_t k, uint16_t* out_x,
                                uint16_t* out_y, void* stream);

/* Description of the last failure on the calling thread; "" if none.  Valid until the next
 * library call on this thread. */
const char* pgti_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PGTI_H */
