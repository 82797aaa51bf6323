// C ABI of the index-batching library (declared in pgti.h): argument checking, ownership of
// device memory, stream ordering.  All arithmetic of the method runs in the kernels of
// series_store.hip, epoch_sort.hip and batch_gather.hip.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <cmath>
#include <new>

#include "pgti_internal.h"

namespace pgti {
namespace {

thread_local char g_error[512] = "";

// Keeps the caller's current device intact around a call.
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t status = hipSuccess;
    explicit DeviceGuard(int device) {
        status = hipGetDevice(&prev);
        if (status == hipSuccess && prev != device) {
            status = hipSetDevice(device);
            switched = (status == hipSuccess);
        }
    }
    ~DeviceGuard() {
        if (switched) (void)hipSetDevice(prev);
    }
};

void free_series(pgti_ctx* c) {
    auto drop = [](auto*& p) {
        if (p) (void)hipFree(p);
        p = nullptr;
    };
    drop(c->d_series);
    drop(c->d_stats);
    drop(c->d_keys[0]);
    drop(c->d_keys[1]);
    drop(c->d_vals[0]);
    drop(c->d_vals[1]);
    drop(c->d_hist);
    drop(c->d_tot);
    drop(c->d_bucket);
    drop(c->d_share);
    drop(c->d_share_next);
    c->loaded = false;
    c->have_share = false;
    c->series_bytes = 0;
}

// Moves the resident store (device buffers, geometry, statistics) of `from` into `to`, whose own
// store must have been freed; `from` is left empty.
void adopt_store(pgti_ctx* to, pgti_ctx* from) {
    auto take = [](auto*& dst, auto*& src) {
        dst = src;
        src = nullptr;
    };
    take(to->d_series, from->d_series);
    take(to->d_stats, from->d_stats);
    for (int k = 0; k < 2; ++k) {
        take(to->d_keys[k], from->d_keys[k]);
        take(to->d_vals[k], from->d_vals[k]);
    }
    take(to->d_hist, from->d_hist);
    take(to->d_tot, from->d_tot);
    take(to->d_bucket, from->d_bucket);
    take(to->d_share, from->d_share);
    take(to->d_share_next, from->d_share_next);
    to->series_bytes = from->series_bytes;
    to->sort_blocks = from->sort_blocks;
    to->mean = from->mean;
    to->stdev = from->stdev;
    to->recip = from->recip;
    to->fast_divide = from->fast_divide;
    to->T = from->T;
    to->N = from->N;
    to->F = from->F;
    to->P = from->P;
    to->Q = from->Q;
    to->B = from->B;
    to->R = from->R;
    to->storage = from->storage;
    to->n_windows = from->n_windows;
    to->path = from->path;
    to->loaded = from->loaded;
    to->have_share = false;
    from->loaded = false;
}

// Temporary device / pinned buffers of one load, released on every exit path.
struct LoadScratch {
    void* pinned[2] = {nullptr, nullptr};
    float* stage[2] = {nullptr, nullptr};
    double* row_acc = nullptr;
    double* stat64 = nullptr;
    hipEvent_t done[2] = {nullptr, nullptr};
    ~LoadScratch() {
        for (int k = 0; k < 2; ++k) {
            if (pinned[k]) (void)hipHostFree(pinned[k]);
            if (stage[k]) (void)hipFree(stage[k]);
            if (done[k]) (void)hipEventDestroy(done[k]);
        }
        if (row_acc) (void)hipFree(row_acc);
        if (stat64) (void)hipFree(stat64);
    }
};

bool host_pointer_is_pinned(const void* p) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();  // an ordinary malloc'd pointer is "invalid value" here: not an error
        return false;
    }
    return attr.type == hipMemoryTypeHost;
}

int check_geometry(int64_t T, int32_t N, int32_t F, int32_t P, int32_t Q, int32_t B, pgti_dtype storage) {
    if (T <= 0 || N <= 0 || F <= 0 || P <= 0 || Q <= 0 || B <= 0)
        return fail(PGTI_ERR_ARG, "T, N, F, P, Q, B must all be positive (got T=%lld N=%d F=%d P=%d Q=%d B=%d)",
                    (long long)T, N, F, P, Q, B);
    if (storage != PGTI_F32 && storage != PGTI_BF16) return fail(PGTI_ERR_ARG, "unknown storage dtype %d", (int)storage);
    if (B > 65535) return fail(PGTI_ERR_RANGE, "batch size %d exceeds 65535", B);
    if (T < static_cast<int64_t>(P) + Q)
        return fail(PGTI_ERR_RANGE, "series of %lld entries holds no window of %d+%d steps", (long long)T, P, Q);
    const int64_t n = T - (static_cast<int64_t>(P) + Q) + 1;
    if (n >= (1ll << 31)) return fail(PGTI_ERR_RANGE, "%lld windows do not fit 32-bit start indices", (long long)n);
    const int64_t R = static_cast<int64_t>(N) * F;
    if ((static_cast<int64_t>(P) + Q) * R >= (1ll << 31))
        return fail(PGTI_ERR_RANGE, "one sample of (P+Q)*N*F = %lld elements exceeds 2^31", (long long)((P + Q) * R));
    return PGTI_OK;
}

SortWorkspace workspace_of(const pgti_ctx* c) {
    return SortWorkspace{{c->d_keys[0], c->d_keys[1]}, {c->d_vals[0], c->d_vals[1]}, c->d_hist,
                         c->d_tot, c->d_bucket, c->bucket_sort_cap, c->sort_key_mask};
}

int check_stats(const float* mean, const float* stdev, int32_t F) {
    for (int32_t f = 0; f < F; ++f) {
        if (!std::isfinite(mean[f]) || !std::isfinite(stdev[f]))
            return fail(PGTI_ERR_STATS, "statistics of feature %d are not finite (mean=%g std=%g)", f, mean[f], stdev[f]);
        if (stdev[f] == 0.0f) return fail(PGTI_ERR_STATS, "standard deviation of feature %d is zero", f);
    }
    return PGTI_OK;
}

// The load itself.  `src` is fp32 [T, N, F_in], on the host or on the device (spec->source_on_device).
int load_impl(pgti_ctx* c, const float* src, const pgti_load_spec* spec) {
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!spec) return fail(PGTI_ERR_ARG, "null load spec");
    if (!src) return fail(PGTI_ERR_ARG, "null series pointer");
    const int64_t T = spec->T;
    const int32_t N = spec->N, F_in = spec->F_in, P = spec->P, Q = spec->Q, B = spec->B;
    const int32_t period = spec->time_of_day_period;
    const pgti_dtype storage = static_cast<pgti_dtype>(spec->storage);
    const bool src_on_device = spec->source_on_device != 0;
    const float* mean = spec->mean;
    const float* stdev = spec->std;
    if (period < 0 || period >= (1 << 24)) return fail(PGTI_ERR_ARG, "time_of_day_period %d not in [0, 2^24)", period);
    if (F_in <= 0) return fail(PGTI_ERR_ARG, "F_in must be positive");
    const bool synth = period > 0;
    const int32_t F = F_in + (synth ? 1 : 0);
    if (int rc = check_geometry(T, N, F, P, Q, B, storage)) return rc;
    const int64_t n = T - (static_cast<int64_t>(P) + Q) + 1;
    int64_t n_train = 0;
    switch (spec->stats_rule) {
        case PGTI_STATS_GIVEN:
            if (!mean || !stdev) return fail(PGTI_ERR_ARG, "PGTI_STATS_GIVEN needs both mean and std");
            if (int rc = check_stats(mean, stdev, F)) return rc;
            break;
        case PGTI_STATS_FEATURE_GLOBAL:
            break;
        case PGTI_STATS_ALG1_TRAIN: {
            if (!(spec->train_fraction > 0.0) || !(spec->train_fraction <= 1.0))
                return fail(PGTI_ERR_ARG, "train_fraction %g not in (0, 1]", spec->train_fraction);
            n_train = static_cast<int64_t>(std::nearbyint(static_cast<double>(n) * spec->train_fraction));
            if (n_train < 1) return fail(PGTI_ERR_RANGE, "training part of %lld windows is empty", (long long)n);
            if (n_train > n) n_train = n;
            break;
        }
        default:
            return fail(PGTI_ERR_ARG, "unknown statistics rule %d", spec->stats_rule);
    }
    const bool need_stats = spec->stats_rule != PGTI_STATS_GIVEN;

    DeviceGuard guard(c->device);
    if (guard.status != hipSuccess) return fail_hip(guard.status, "hipSetDevice");
    hipStream_t ws = c->work_stream;
    PGTI_HIP_TRY(hipStreamSynchronize(ws));
    // A source that lives on the device may still be being written by work the caller enqueued on
    // any of its streams: wait for all of it before the first read (the load is synchronous anyway).
    if (src_on_device) PGTI_HIP_TRY(hipDeviceSynchronize());

    // The new store is built beside the old one and replaces it only when everything has succeeded:
    // a failed load leaves the context exactly as it was.  The new store is released on every early return.
    pgti_ctx fresh_store;
    pgti_ctx* nx = &fresh_store;
    struct Release {
        pgti_ctx* store;
        ~Release() {
            if (store) free_series(store);
        }
    } release{nx};

    const int64_t R = static_cast<int64_t>(N) * F, R_in = static_cast<int64_t>(N) * F_in;
    const size_t elems = static_cast<size_t>(T) * R;
    const size_t store_bytes = (storage == PGTI_F32) ? 4 : 2;

    auto alloc = [&](auto** p, size_t bytes) -> int {
        hipError_t e = hipMalloc(reinterpret_cast<void**>(p), bytes < 256 ? 256 : bytes);
        if (e == hipErrorOutOfMemory) {
            (void)hipGetLastError();
            free_series(nx);
            return fail(PGTI_ERR_OOM, "device allocation of %zu bytes failed", bytes);
        }
        if (e != hipSuccess) {
            free_series(nx);
            return fail_hip(e, "hipMalloc");
        }
        return PGTI_OK;
    };

    const uint32_t nblk = static_cast<uint32_t>((n + kSortTile - 1) / kSortTile);
    if (int rc = alloc(&nx->d_series, elems * store_bytes)) return rc;
    if (int rc = alloc(&nx->d_stats, sizeof(float) * 3 * F)) return rc;
    if (int rc = alloc(&nx->d_keys[0], sizeof(uint64_t) * n)) return rc;
    if (int rc = alloc(&nx->d_keys[1], sizeof(uint64_t) * n)) return rc;
    if (int rc = alloc(&nx->d_vals[0], sizeof(int32_t) * n)) return rc;
    if (int rc = alloc(&nx->d_vals[1], sizeof(int32_t) * n)) return rc;
    if (int rc = alloc(&nx->d_hist, sizeof(uint32_t) * 256 * nblk)) return rc;
    if (int rc = alloc(&nx->d_tot, sizeof(uint32_t) * 256)) return rc;
    if (int rc = alloc(&nx->d_bucket, sizeof(uint32_t) * kSortBucketWords)) return rc;
    PGTI_HIP_TRY(hipMemsetAsync(nx->d_bucket, 0, sizeof(uint32_t) * kSortBucketWords, ws));
    if (int rc = alloc(&nx->d_share, sizeof(int32_t) * n)) return rc;
    if (int rc = alloc(&nx->d_share_next, sizeof(int32_t) * n)) return rc;
    nx->series_bytes = elems * store_bytes;
    nx->sort_blocks = nblk;

    // A device source is taken in one piece.  A host source moves in chunks of about 64 MiB of fp32,
    // a multiple of 4 rows so that every chunk starts on a 16-byte boundary whatever R is.
    int64_t chunk_rows = (64ll << 20) / (R * 4);
    chunk_rows = (chunk_rows / 4) * 4;
    if (chunk_rows < 4) chunk_rows = 4;
    if (src_on_device) chunk_rows = T;
    const size_t chunk_bytes_in = static_cast<size_t>(chunk_rows) * R_in * 4;

    LoadScratch tmp;
    const bool src_pinned = !src_on_device && host_pointer_is_pinned(src);
    const bool via_pinned_staging = !src_on_device && !src_pinned;
    // A host chunk lands in a device staging buffer unless it can go straight into the fp32 store.
    const bool via_device_staging = !src_on_device && (storage == PGTI_BF16 || synth);
    for (int k = 0; k < 2; ++k) {
        PGTI_HIP_TRY(hipEventCreateWithFlags(&tmp.done[k], hipEventDisableTiming));
        if (via_pinned_staging) {
            hipError_t e = hipHostMalloc(&tmp.pinned[k], chunk_bytes_in, hipHostMallocDefault);
            if (e != hipSuccess) {
                (void)hipGetLastError();
                free_series(nx);
                return fail(PGTI_ERR_OOM, "pinned staging allocation of %zu bytes failed", chunk_bytes_in);
            }
        }
        if (via_device_staging)
            if (int rc = alloc(&tmp.stage[k], chunk_bytes_in)) return rc;
    }
    if (need_stats) {
        if (int rc = alloc(&tmp.row_acc, sizeof(double) * static_cast<size_t>(T) * F)) return rc;
        if (int rc = alloc(&tmp.stat64, sizeof(double) * F)) return rc;
    }

    // Sweep 0 moves the data (and sums values if statistics are wanted); sweep 1, only with
    // statistics, sums squared deviations from the mean.  Statistics always see fp32 values: with
    // fp32 storage the finished resident rows, with bf16 storage the source chunk (the time-of-day
    // channel synthesised on the fly); the bf16 rounding happens in the last sweep.  Every chunk is
    // ONE kernel: it writes the resident rows and takes the row sums from the same registers.
    const int sweeps = need_stats ? 2 : 1;
    double* const row_acc = need_stats ? tmp.row_acc : nullptr;
    for (int sweep = 0; sweep < sweeps; ++sweep) {
        const bool last_sweep = (sweep == sweeps - 1);
        const double* const mean64 = (need_stats && sweep == 1) ? tmp.stat64 : nullptr;
        if (storage == PGTI_F32 && sweep == 1) {
            // the whole resident series in one launch
            PGTI_HIP_TRY(launch_ingest_rows(static_cast<const float*>(nx->d_series), T, N, F, F, 0, 0, nullptr, false,
                                            mean64, row_acc, ws));
        } else {
            int slot = 0;
            bool slot_busy[2] = {false, false};
            for (int64_t row0 = 0; row0 < T; row0 += chunk_rows, slot ^= 1) {
                const int64_t rows = (T - row0 < chunk_rows) ? (T - row0) : chunk_rows;
                const size_t off = static_cast<size_t>(row0) * R, off_in = static_cast<size_t>(row0) * R_in;
                const size_t cnt_in = static_cast<size_t>(rows) * R_in;
                float* resident32 = static_cast<float*>(nx->d_series) + off;        // fp32 storage
                uint16_t* resident16 = static_cast<uint16_t*>(nx->d_series) + off;  // bf16 storage

                // the source chunk on the device
                const float* src_chunk = nullptr;
                if (src_on_device) {
                    src_chunk = src + off_in;
                } else {
                    if (slot_busy[slot]) PGTI_HIP_TRY(hipEventSynchronize(tmp.done[slot]));
                    float* dst = via_device_staging ? tmp.stage[slot] : resident32;
                    const void* from = src + off_in;
                    if (via_pinned_staging) {
                        memcpy(tmp.pinned[slot], src + off_in, cnt_in * 4);
                        from = tmp.pinned[slot];
                    }
                    PGTI_HIP_TRY(hipMemcpyAsync(dst, from, cnt_in * 4, hipMemcpyHostToDevice, ws));
                    src_chunk = dst;
                }

                void* out = nullptr;
                if (storage == PGTI_F32) {
                    if (src_chunk != resident32) out = resident32;  // else the copy has put the rows in place
                } else if (last_sweep) {
                    out = resident16;
                }
                PGTI_HIP_TRY(launch_ingest_rows(src_chunk, rows, N, F, F_in, period, row0, out, storage == PGTI_BF16,
                                                mean64, row_acc, ws));
                PGTI_HIP_TRY(hipEventRecord(tmp.done[slot], ws));
                slot_busy[slot] = true;
            }
        }
        if (need_stats) {
            // mean after sweep 0 (kept in fp64 on the device for sweep 1), std after sweep 1
            float* out32 = nx->d_stats + (sweep == 0 ? 0 : F);
            if (spec->stats_rule == PGTI_STATS_ALG1_TRAIN)
                PGTI_HIP_TRY(launch_reduce_rows_alg1(tmp.row_acc, F, n_train, P,
                                                     static_cast<double>(n_train) * P * static_cast<double>(R),
                                                     sweep == 1, tmp.stat64, out32, ws));
            else
                PGTI_HIP_TRY(launch_reduce_rows(tmp.row_acc, T, N, F, sweep == 1, tmp.stat64, out32, ws));
        }
        PGTI_HIP_TRY(hipStreamSynchronize(ws));
    }

    nx->mean.assign(F, 0.0f);
    nx->stdev.assign(F, 1.0f);
    if (need_stats) {
        PGTI_HIP_TRY(hipMemcpy(nx->mean.data(), nx->d_stats, sizeof(float) * F, hipMemcpyDeviceToHost));
        PGTI_HIP_TRY(hipMemcpy(nx->stdev.data(), nx->d_stats + F, sizeof(float) * F, hipMemcpyDeviceToHost));
        if (int rc = check_stats(nx->mean.data(), nx->stdev.data(), F)) {
            free_series(nx);
            return rc;
        }
    } else {
        memcpy(nx->mean.data(), mean, sizeof(float) * F);
        memcpy(nx->stdev.data(), stdev, sizeof(float) * F);
        PGTI_HIP_TRY(hipMemcpy(nx->d_stats, nx->mean.data(), sizeof(float) * F, hipMemcpyHostToDevice));
        PGTI_HIP_TRY(hipMemcpy(nx->d_stats + F, nx->stdev.data(), sizeof(float) * F, hipMemcpyHostToDevice));
    }

    // Reciprocals for the gather's fast division: 1/sigma in fp64 rounded once to fp32 is the
    // correctly rounded fp32 reciprocal (53 >= 2*24 + 2 bits).  The fast path needs every sigma's
    // biased exponent in [95, 159]; otherwise the kernels divide the ordinary way.
    nx->recip.assign(F, 1.0f);
    nx->fast_divide = true;
    for (int32_t f = 0; f < F; ++f) {
        uint32_t bits;
        memcpy(&bits, &nx->stdev[f], 4);
        const uint32_t expo = (bits >> 23) & 0xFFu;
        if (expo < 95u || expo > 159u) nx->fast_divide = false;
        nx->recip[f] = static_cast<float>(1.0 / static_cast<double>(nx->stdev[f]));
    }
    PGTI_HIP_TRY(hipMemcpy(nx->d_stats + 2 * F, nx->recip.data(), sizeof(float) * F, hipMemcpyHostToDevice));

    nx->T = T;
    nx->N = N;
    nx->F = F;
    nx->P = P;
    nx->Q = Q;
    nx->B = B;
    nx->R = R;
    nx->storage = storage;
    nx->n_windows = n;
    const bool quad_ok = ((static_cast<int64_t>(P) * R) % 4 == 0) && ((static_cast<int64_t>(Q) * R) % 4 == 0);
    nx->path = quad_ok ? GatherPath::kQuads : GatherPath::kScalar;
    nx->loaded = true;
    nx->have_share = false;

    // Success: batch builds enqueued through this context may still read the old series; wait for
    // them, free it, and adopt the new store.
    for (int k = 0; k < c->n_tracked; ++k) PGTI_HIP_TRY(hipStreamSynchronize(c->tracked[k].stream));
    c->n_tracked = 0;
    free_series(c);
    adopt_store(c, nx);
    release.store = nullptr;
    return PGTI_OK;
}

}  // namespace

int fail(int status, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return status;
}

int fail_hip(hipError_t e, const char* what) {
    (void)hipGetLastError();
    snprintf(g_error, sizeof(g_error), "HIP error %d (%s) in %s", (int)e, hipGetErrorString(e), what);
    return e == hipErrorOutOfMemory ? PGTI_ERR_OOM : PGTI_ERR_HIP;
}

void clear_error() { g_error[0] = 0; }

}  // namespace pgti

using namespace pgti;

extern "C" {

int pgti_create(pgti_ctx** out, int device) {
    g_error[0] = 0;
    if (!out) return fail(PGTI_ERR_ARG, "null output handle");
    *out = nullptr;
    int count = 0;
    PGTI_HIP_TRY(hipGetDeviceCount(&count));
    if (device < 0 || device >= count) return fail(PGTI_ERR_ARG, "device %d not in [0, %d)", device, count);
    pgti_ctx* c = new (std::nothrow) pgti_ctx();
    if (!c) return fail(PGTI_ERR_OOM, "host allocation failed");
    c->device = device;
    c->bucket_sort_cap = kBucketSortKeys;
    DeviceGuard guard(device);
    hipError_t e = guard.status;
    // Set-up of the allocation-free epoch order: resolve this device's copy of its scratch array now,
    // so that the call itself never has to (it may run where symbol look-ups are unwelcome).
    void* static_scratch = nullptr;
    if (e == hipSuccess) e = static_sort_scratch(device, &static_scratch);
    if (e == hipSuccess) e = hipStreamCreateWithFlags(&c->work_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_share_ready, hipEventDisableTiming);
    for (int k = 0; k < kMaxTrackedStreams && e == hipSuccess; ++k) {
        c->tracked[k].stream = nullptr;
        c->tracked[k].event = nullptr;
        e = hipEventCreateWithFlags(&c->tracked[k].event, hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        int rc = fail_hip(e, "creating stream/events");
        pgti_destroy(c);
        return rc;
    }
    *out = c;
    return PGTI_OK;
}

void pgti_destroy(pgti_ctx* c) {
    if (!c) return;
    DeviceGuard guard(c->device);
    if (c->work_stream) (void)hipStreamSynchronize(c->work_stream);
    for (int k = 0; k < c->n_tracked; ++k) (void)hipStreamSynchronize(c->tracked[k].stream);
    free_series(c);
    for (int k = 0; k < kMaxTrackedStreams; ++k)
        if (c->tracked[k].event) (void)hipEventDestroy(c->tracked[k].event);
    if (c->ev_share_ready) (void)hipEventDestroy(c->ev_share_ready);
    if (c->work_stream) (void)hipStreamDestroy(c->work_stream);
    delete c;
}

static pgti_load_spec basic_spec(int64_t T, int32_t N, int32_t F, int32_t P, int32_t Q, int32_t B, pgti_dtype storage,
                                 const float* mean, const float* std, int on_device) {
    pgti_load_spec spec;
    memset(&spec, 0, sizeof(spec));
    spec.T = T;
    spec.N = N;
    spec.F_in = F;
    spec.P = P;
    spec.Q = Q;
    spec.B = B;
    spec.storage = storage;
    spec.source_on_device = on_device;
    spec.stats_rule = (mean || std) ? PGTI_STATS_GIVEN : PGTI_STATS_FEATURE_GLOBAL;
    spec.train_fraction = 0.70;
    spec.mean = mean;
    spec.std = std;
    return spec;
}

int pgti_load_series(pgti_ctx* c, const float* host_series, int64_t T, int32_t N, int32_t F, int32_t P,
                     int32_t Q, int32_t B, pgti_dtype storage, const float* mean, const float* std) {
    g_error[0] = 0;
    if ((mean == nullptr) != (std == nullptr)) return fail(PGTI_ERR_ARG, "pass both mean and std, or neither");
    const pgti_load_spec spec = basic_spec(T, N, F, P, Q, B, storage, mean, std, 0);
    return load_impl(c, host_series, &spec);
}

int pgti_load_series_device(pgti_ctx* c, const float* device_series, int64_t T, int32_t N, int32_t F,
                            int32_t P, int32_t Q, int32_t B, pgti_dtype storage, const float* mean,
                            const float* std) {
    g_error[0] = 0;
    if ((mean == nullptr) != (std == nullptr)) return fail(PGTI_ERR_ARG, "pass both mean and std, or neither");
    const pgti_load_spec spec = basic_spec(T, N, F, P, Q, B, storage, mean, std, 1);
    return load_impl(c, device_series, &spec);
}

int pgti_load_series_ex(pgti_ctx* c, const float* series, const pgti_load_spec* spec) {
    g_error[0] = 0;
    return load_impl(c, series, spec);
}

int pgti_set_sort_test_hooks(pgti_ctx* c, uint32_t bucket_cap, uint32_t key_bits) {
    g_error[0] = 0;
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (bucket_cap >= kBucketSortKeys) return fail(PGTI_ERR_ARG, "bucket_cap %u not in [0, %u)", bucket_cap, kBucketSortKeys);
    if (key_bits > 64) return fail(PGTI_ERR_ARG, "key_bits %u not in [0, 64]", key_bits);
    c->bucket_sort_cap = bucket_cap ? bucket_cap : kBucketSortKeys;
    c->sort_key_mask = (key_bits == 0 || key_bits == 64) ? ~0ull : ~((1ull << (64 - key_bits)) - 1ull);
    return PGTI_OK;
}

int pgti_get_stats(pgti_ctx* c, float* mean_out, float* std_out) {
    g_error[0] = 0;
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!c->loaded) return fail(PGTI_ERR_STATE, "no series loaded");
    if (mean_out) memcpy(mean_out, c->mean.data(), sizeof(float) * c->F);
    if (std_out) memcpy(std_out, c->stdev.data(), sizeof(float) * c->F);
    return PGTI_OK;
}

int pgti_epoch_indices_ex(pgti_ctx* c, const pgti_epoch_spec* spec, int64_t* n_share) {
    g_error[0] = 0;
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!spec) return fail(PGTI_ERR_ARG, "null epoch spec");
    if (!c->loaded) return fail(PGTI_ERR_STATE, "no series loaded");
    if (spec->order != PGTI_ORDER_SHUFFLE && spec->order != PGTI_ORDER_SEQUENTIAL &&
        spec->order != PGTI_ORDER_BATCH_SHUFFLE)
        return fail(PGTI_ERR_ARG, "unknown epoch order %d", spec->order);
    if (spec->world == 0) return fail(PGTI_ERR_RANGE, "world must be at least 1");
    if (spec->rank >= spec->world) return fail(PGTI_ERR_RANGE, "rank %u not in [0, %u)", spec->rank, spec->world);
    const int64_t first_start = spec->first_start;
    if (first_start < 0 || first_start > c->n_windows)
        return fail(PGTI_ERR_RANGE, "first_start %lld not in [0, %lld]", (long long)first_start, (long long)c->n_windows);
    const int64_t n_starts = spec->n_starts < 0 ? c->n_windows - first_start : spec->n_starts;
    if (n_starts > c->n_windows - first_start)
        return fail(PGTI_ERR_RANGE, "starts [%lld, %lld) exceed the %lld windows", (long long)first_start,
                    (long long)(first_start + n_starts), (long long)c->n_windows);
    DeviceGuard guard(c->device);
    if (guard.status != hipSuccess) return fail_hip(guard.status, "hipSetDevice");

    const uint64_t n = static_cast<uint64_t>(n_starts);
    const uint64_t lo = (static_cast<uint64_t>(spec->rank) * n) / spec->world;  // < 2^32 * 2^31: no overflow
    const uint64_t hi = ((static_cast<uint64_t>(spec->rank) + 1) * n) / spec->world;
    const uint32_t len = static_cast<uint32_t>(hi - lo);

    // The new order is computed into a staging buffer, so it may run while batch builds of the
    // current epoch still read the share; only the short copy that publishes it (below) is ordered
    // behind them.  The builds keep reading one fixed address from epoch to epoch.
    hipStream_t ws = c->work_stream;
    int32_t* share_out = c->d_share_next;
    if (spec->order == PGTI_ORDER_SHUFFLE) {
        SortPlan plan{static_cast<uint32_t>(n), 0, 1, share_out, static_cast<uint32_t>(lo),
                      static_cast<uint32_t>(hi), static_cast<int32_t>(first_start)};
        PGTI_HIP_TRY(launch_sorted_order(workspace_of(c), spec->seed, spec->epoch, plan, ws));
    } else if (spec->order == PGTI_ORDER_SEQUENTIAL) {
        PGTI_HIP_TRY(launch_sequential_order(share_out, len, static_cast<int32_t>(first_start + lo), ws));
    } else {
        // Order of the full batches of the partition [lo, hi): keys on the position of each batch's
        // first element; the sorted batch numbers pass through d_vals[0], then expand to starts.
        const uint32_t n_full = len / static_cast<uint32_t>(c->B);
        SortPlan plan{n_full, lo, static_cast<uint64_t>(c->B), c->d_vals[0], 0, n_full, 0};
        PGTI_HIP_TRY(launch_sorted_order(workspace_of(c), spec->seed, spec->epoch, plan, ws));
        PGTI_HIP_TRY(launch_expand_batches(c->d_vals[0], n_full, static_cast<uint32_t>(c->B),
                                           static_cast<int32_t>(first_start + lo), share_out, len, ws));
    }
    // Publish: the share is overwritten only after every batch build that was enqueued through this
    // context since the last index generation has finished reading it.
    for (int k = 0; k < c->n_tracked; ++k) {
        PGTI_HIP_TRY(hipEventRecord(c->tracked[k].event, c->tracked[k].stream));
        PGTI_HIP_TRY(hipStreamWaitEvent(ws, c->tracked[k].event, 0));
    }
    c->n_tracked = 0;
    if (len > 0)
        PGTI_HIP_TRY(hipMemcpyAsync(c->d_share, share_out, sizeof(int32_t) * len, hipMemcpyDeviceToDevice, ws));
    PGTI_HIP_TRY(hipEventRecord(c->ev_share_ready, ws));
    c->share_lo = static_cast<int64_t>(lo);
    c->share_hi = static_cast<int64_t>(hi);
    c->have_share = true;
    c->share_consecutive = (spec->order != PGTI_ORDER_SHUFFLE);
    if (n_share) *n_share = static_cast<int64_t>(hi - lo);
    return PGTI_OK;
}

int pgti_epoch_indices(pgti_ctx* c, uint64_t seed, uint64_t epoch, uint32_t rank, uint32_t world,
                       int64_t* n_share) {
    pgti_epoch_spec spec;
    memset(&spec, 0, sizeof(spec));
    spec.order = PGTI_ORDER_SHUFFLE;
    spec.first_start = 0;
    spec.n_starts = -1;
    spec.seed = seed;
    spec.epoch = epoch;
    spec.rank = rank;
    spec.world = world;
    return pgti_epoch_indices_ex(c, &spec, n_share);
}

int64_t pgti_get_indices(pgti_ctx* c, int32_t* host_out, int64_t capacity) {
    g_error[0] = 0;
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!c->loaded || !c->have_share) return fail(PGTI_ERR_STATE, "no epoch indices generated");
    const int64_t len = c->share_hi - c->share_lo;
    if (len > 0 && (!host_out || capacity < len))
        return fail(PGTI_ERR_ARG, "share of %lld starts does not fit capacity %lld", (long long)len, (long long)capacity);
    DeviceGuard guard(c->device);
    if (guard.status != hipSuccess) return fail_hip(guard.status, "hipSetDevice");
    PGTI_HIP_TRY(hipStreamSynchronize(c->work_stream));
    if (len > 0) PGTI_HIP_TRY(hipMemcpy(host_out, c->d_share, sizeof(int32_t) * len, hipMemcpyDeviceToHost));
    return len;
}

int64_t pgti_num_batches(pgti_ctx* c) {
    g_error[0] = 0;
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!c->loaded || !c->have_share) return fail(PGTI_ERR_STATE, "no epoch indices generated");
    const int64_t len = c->share_hi - c->share_lo;
    return (len + c->B - 1) / c->B;
}

// Common part of the single- and multi-batch builds: checks, stream ordering, launches.
static int64_t build_range(pgti_ctx* c, int64_t first_batch, int64_t k, void* out_x, void* out_y, bool out_bf16,
                           void* stream) {
    if (!c) return fail(PGTI_ERR_ARG, "null context");
    if (!c->loaded) return fail(PGTI_ERR_STATE, "no series loaded");
    if (!c->have_share) return fail(PGTI_ERR_STATE, "no epoch indices generated");
    if (!out_x || !out_y) return fail(PGTI_ERR_ARG, "null output pointer");
    if ((reinterpret_cast<uintptr_t>(out_x) | reinterpret_cast<uintptr_t>(out_y)) & 15u)
        return fail(PGTI_ERR_ARG, "outputs must be 16-byte aligned");
    const int64_t len = c->share_hi - c->share_lo;
    const int64_t nb = (len + c->B - 1) / c->B;
    if (k < 1) return fail(PGTI_ERR_RANGE, "batch count %lld must be at least 1", (long long)k);
    if (first_batch < 0 || first_batch >= nb || k > nb - first_batch)
        return fail(PGTI_ERR_RANGE, "batches [%lld, %lld) not in [0, %lld)", (long long)first_batch,
                    (long long)(first_batch + k), (long long)nb);
    const int64_t first = first_batch * c->B;
    const int64_t last = (first + k * c->B < len) ? (first + k * c->B) : len;
    const int64_t count = last - first;

    DeviceGuard guard(c->device);
    if (guard.status != hipSuccess) return fail_hip(guard.status, "hipSetDevice");
    hipStream_t s = static_cast<hipStream_t>(stream);

    // First build on this stream since the last sort: make the stream wait for the share.
    bool known = false;
    for (int t = 0; t < c->n_tracked; ++t) known = known || (c->tracked[t].stream == s);
    if (!known) {
        int slot = c->n_tracked;
        if (c->n_tracked == kMaxTrackedStreams) {
            // More streams than slots: finish the builds of the oldest on the host and reuse its slot.
            PGTI_HIP_TRY(hipStreamSynchronize(c->tracked[0].stream));
            slot = 0;
        } else {
            ++c->n_tracked;
        }
        PGTI_HIP_TRY(hipStreamWaitEvent(s, c->ev_share_ready, 0));
        c->tracked[slot].stream = s;
    }

    // Samples are consecutive in the share and in the outputs, so several batches are one launch
    // with more samples; the grid's sample dimension holds at most 65,535.
    const int64_t x_stride = static_cast<int64_t>(c->P) * c->R, y_stride = static_cast<int64_t>(c->Q) * c->R;
    const int64_t max_part = (65535 / c->B) * static_cast<int64_t>(c->B);  // whole batches per launch
    for (int64_t done = 0; done < count; done += max_part) {
        const int32_t part = static_cast<int32_t>((count - done < max_part) ? (count - done) : max_part);
        const size_t out_elem = out_bf16 ? 2 : 4;
        PGTI_HIP_TRY(launch_batch_gather(c, c->d_share + first + done, part,
                                         static_cast<char*>(out_x) + done * x_stride * out_elem,
                                         static_cast<char*>(out_y) + done * y_stride * out_elem, out_bf16, s));
    }
    return count;
}

int pgti_build_batch(pgti_ctx* c, int64_t batch_no, float* out_x, float* out_y, void* stream) {
    g_error[0] = 0;
    return static_cast<int>(build_range(c, batch_no, 1, out_x, out_y, false, stream));
}

int64_t pgti_build_batches(pgti_ctx* c, int64_t first_batch, int32_t k, float* out_x, float* out_y,
                           void* stream) {
    g_error[0] = 0;
    return build_range(c, first_batch, k, out_x, out_y, false, stream);
}

int64_t pgti_build_batches_bf16(pgti_ctx* c, int64_t first_batch, int32_t k, uint16_t* out_x, uint16_t* out_y,
                                void* stream) {
    g_error[0] = 0;
    return build_range(c, first_batch, k, out_x, out_y, true, stream);
}

const char* pgti_last_error(void) { return g_error; }

}  // extern "C"
