/*
 * CPU oracle for index-batched snapshot construction (PGT-I, arXiv 2507.11683).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, single-threaded
 * statement of what the hot path computes, written so that each function can be checked
 * against the paper by eye.  Only the tests, the smoke check and the CPU-baseline leg of
 * the benchmark may call it.  It shares no code, header, table or helper with the HIP
 * library and neither includes the other.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC  (no FMA contraction, so
 * every fp32 operation below is one IEEE-754 binary32 round-to-nearest-even operation).
 *
 * Notation follows the paper: a series `data` of `entries` x `nodes` x `features`
 * (here T x N x F, row-major, F fastest); `horizon` is split into P (input length) and
 * Q (target length); `start` is the graph ID of the first entry of a snapshot.
 *
 * Pins (see tests, all CPU-only):
 *   window count / Eq. 1 / Eq. 2 ....... Table 1 "size after preprocessing" column
 *   windows as slices ................... Sec. 4.1 worked example (horizon 3), numpy slicing,
 *                                         numpy sliding_window_view, Algorithm 1 brute force
 *   standardize ......................... exact rational arithmetic rounded once per operation
 *   key mixer ........................... published splitmix64 stream from state 0
 *   epoch order ......................... permutation/coverage invariants, numpy lexsort
 *   bf16 rounding ....................... an independent library conversion (torch)
 *   series statistics ................... numpy mean/std in fp64
 * The particular permutation depends on how (seed, epoch, i) are combined into a key; the
 * paper fixes no generator, so that combination is this build's own reading: parity unpinned
 * with respect to the paper for that one choice (it is pinned GPU <-> oracle bit for bit).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORACLE_OK 0
#define ORACLE_ERR_ARG (-1)

/* ------------------------------------------------------------------------------------------
 * Counting (Eq. 1, Eq. 2).
 * ---------------------------------------------------------------------------------------- */

/* Number of valid window placements.  Eq. 1 and Eq. 2 both use entries - (2*horizon - 1);
 * with separate input/target lengths that is T - (P + Q) + 1.  Non-positive -> 0. */
int64_t oracle_window_count(int64_t T, int64_t P, int64_t Q) {
    int64_t n = T - (P + Q) + 1;
    return n > 0 ? n : 0;
}

/* Eq. 1: element count of the materialised x and y arrays,
 * 2 * [(entries - (2*horizon - 1)) * horizon * nodes * features]. */
int64_t oracle_eq1_materialized_elements(int64_t entries, int64_t horizon, int64_t nodes,
                                         int64_t features) {
    return 2 * ((entries - (2 * horizon - 1)) * horizon * nodes * features);
}

/* Eq. 2: element count held by index-batching: one copy of the data plus one index per
 * window, entries*nodes*features + (entries - (2*horizon - 1)). */
int64_t oracle_eq2_index_batching_elements(int64_t entries, int64_t horizon, int64_t nodes,
                                           int64_t features) {
    return entries * nodes * features + (entries - (2 * horizon - 1));
}

/* ------------------------------------------------------------------------------------------
 * Epoch order (Sec. 4.2: shuffle at the start of each epoch, then partition by the number of
 * workers).  The shuffle is defined as: sort the starts 0..n-1 by (key_i, i) ascending.
 * ---------------------------------------------------------------------------------------- */

/* The splitmix64 output function (Steele, Lea, Flood 2014; Vigna's public-domain reference):
 * z ^= z>>30; z *= 0xBF58476D1CE4E5B9; z ^= z>>27; z *= 0x94D049BB133111EB; z ^= z>>31. */
uint64_t oracle_mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * UINT64_C(0xBF58476D1CE4E5B9);
    z = (z ^ (z >> 27)) * UINT64_C(0x94D049BB133111EB);
    return z ^ (z >> 31);
}

/* The classic splitmix64 stream: state += gamma; return mix(state).  Only used to pin
 * oracle_mix64 against the published first outputs for state 0. */
uint64_t oracle_splitmix64_next(uint64_t* state) {
    *state += UINT64_C(0x9E3779B97F4A7C15);
    return oracle_mix64(*state);
}

/* key_i = M((h1 ^ i) + g), h1 = M((h0 ^ epoch) + g), h0 = M(seed + g), g the golden gamma.
 * Each argument passes through one full mixing round before the next is folded in. */
uint64_t oracle_key(uint64_t seed, uint64_t epoch, uint64_t i) {
    const uint64_t g = UINT64_C(0x9E3779B97F4A7C15);
    uint64_t h0 = oracle_mix64(seed + g);
    uint64_t h1 = oracle_mix64((h0 ^ epoch) + g);
    return oracle_mix64((h1 ^ i) + g);
}

/* The keys of the first n starts of an epoch, keys_out[i] = key(seed, epoch, i): the list that
 * oracle_sort_pairs orders into the epoch's permutation. */
int oracle_keys(uint64_t seed, uint64_t epoch, int64_t n, uint64_t* keys_out) {
    if (n < 0 || (n > 0 && !keys_out)) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) keys_out[i] = oracle_key(seed, epoch, (uint64_t)i);
    return ORACLE_OK;
}

typedef struct {
    uint64_t key;
    int32_t idx;
} oracle_pair;

static int pair_less(const void* a, const void* b) {
    const oracle_pair* pa = (const oracle_pair*)a;
    const oracle_pair* pb = (const oracle_pair*)b;
    if (pa->key != pb->key) return pa->key < pb->key ? -1 : 1;
    if (pa->idx != pb->idx) return pa->idx < pb->idx ? -1 : 1; /* equal keys: lower start first */
    return 0;
}

/* Sort n (key, index) pairs ascending by key, ties by index: a total order, so any
 * comparison sort gives the one answer.  perm_out receives the indices in sorted order. */
int oracle_sort_pairs(const uint64_t* keys, int64_t n, int32_t* perm_out) {
    if (n < 0 || n > INT32_MAX || (n > 0 && (!keys || !perm_out))) return ORACLE_ERR_ARG;
    if (n == 0) return ORACLE_OK;
    oracle_pair* pairs = (oracle_pair*)malloc((size_t)n * sizeof(oracle_pair));
    if (!pairs) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        pairs[i].key = keys[i];
        pairs[i].idx = (int32_t)i;
    }
    qsort(pairs, (size_t)n, sizeof(oracle_pair), pair_less);
    for (int64_t i = 0; i < n; ++i) perm_out[i] = pairs[i].idx;
    free(pairs);
    return ORACLE_OK;
}

/* The whole epoch's order of starts: perm = argsort of (key_i, i), i in [0, n). */
int oracle_epoch_perm(uint64_t seed, uint64_t epoch, int64_t n, int32_t* perm_out) {
    if (n < 0 || n > INT32_MAX || (n > 0 && !perm_out)) return ORACLE_ERR_ARG;
    if (n == 0) return ORACLE_OK;
    uint64_t* keys = (uint64_t*)malloc((size_t)n * sizeof(uint64_t));
    if (!keys) return ORACLE_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) keys[i] = oracle_key(seed, epoch, (uint64_t)i);
    int rc = oracle_sort_pairs(keys, n, perm_out);
    free(keys);
    return rc;
}

/* Partition by number of workers: rank r of `world` owns perm[lo:hi),
 * lo = floor(r*n/world), hi = floor((r+1)*n/world).  Nothing padded, nothing dropped. */
int oracle_rank_share(int64_t n, int64_t rank, int64_t world, int64_t* lo, int64_t* hi) {
    if (n < 0 || world <= 0 || rank < 0 || rank >= world || !lo || !hi) return ORACLE_ERR_ARG;
    *lo = (rank * n) / world;
    *hi = ((rank + 1) * n) / world;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * Other epoch orders and start ranges.
 *
 * Range: Sec. 3.1 splits the windows 70/10/20 into train, validation and test, and Algorithm 1
 * takes x_train as the leading part of the stacked windows, so a split is a contiguous range
 * of starts [first_start, first_start + n_starts).  Positions inside the range are 0..n_starts-1.
 *
 * order 0, global shuffle (Sec. 4.2): positions sorted by (key(seed, epoch, position), position),
 *          the rank takes its contiguous slice of that order.
 * order 1, sequential (validation / test passes, and the unshuffled reading of Algorithm 1):
 *          the rank takes its contiguous slice [lo, hi) of the positions in time order.
 * order 2, batch-level shuffle (Sec. 5.4: a fixed data partition per worker; the order of the
 *          batches is shuffled while the data inside a batch stays fixed): the rank's partition
 *          is the same slice [lo, hi) as in order 1, every epoch; it is cut into consecutive
 *          batches of B positions; the full batches are visited in the order of ascending
 *          (key(seed, epoch, position of the batch's first element), batch number); a short
 *          remainder batch, if any, comes last so that only the last batch of a share is short.
 * Every returned value is first_start + position.
 * ---------------------------------------------------------------------------------------- */
int oracle_epoch_indices_ex(int order, int64_t n_windows, int64_t first_start, int64_t n_starts,
                            int64_t B, uint64_t seed, uint64_t epoch, int64_t rank, int64_t world,
                            int32_t* out, int64_t* n_out) {
    if (!n_out || first_start < 0 || n_starts < 0 || first_start + n_starts > n_windows || B <= 0)
        return ORACLE_ERR_ARG;
    int64_t lo, hi;
    if (oracle_rank_share(n_starts, rank, world, &lo, &hi) != ORACLE_OK) return ORACLE_ERR_ARG;
    int64_t len = hi - lo;
    *n_out = len;
    if (len > 0 && !out) return ORACLE_ERR_ARG;
    if (order == 0) {
        int32_t* perm = (int32_t*)malloc((size_t)(n_starts > 0 ? n_starts : 1) * sizeof(int32_t));
        if (!perm) return ORACLE_ERR_ARG;
        int rc = oracle_epoch_perm(seed, epoch, n_starts, perm);
        for (int64_t i = 0; rc == ORACLE_OK && i < len; ++i) out[i] = (int32_t)(first_start + perm[lo + i]);
        free(perm);
        return rc;
    }
    if (order == 1) {
        for (int64_t i = 0; i < len; ++i) out[i] = (int32_t)(first_start + lo + i);
        return ORACLE_OK;
    }
    if (order == 2) {
        int64_t n_full = len / B;
        uint64_t* keys = (uint64_t*)malloc((size_t)(n_full > 0 ? n_full : 1) * sizeof(uint64_t));
        int32_t* batch_order = (int32_t*)malloc((size_t)(n_full > 0 ? n_full : 1) * sizeof(int32_t));
        if (!keys || !batch_order) { free(keys); free(batch_order); return ORACLE_ERR_ARG; }
        for (int64_t b = 0; b < n_full; ++b) keys[b] = oracle_key(seed, epoch, (uint64_t)(lo + b * B));
        int rc = oracle_sort_pairs(keys, n_full, batch_order);
        for (int64_t i = 0; rc == ORACLE_OK && i < n_full; ++i)
            for (int64_t j = 0; j < B; ++j)
                out[i * B + j] = (int32_t)(first_start + lo + (int64_t)batch_order[i] * B + j);
        for (int64_t i = n_full * B; rc == ORACLE_OK && i < len; ++i) /* the short remainder batch */
            out[i] = (int32_t)(first_start + lo + i);
        free(keys);
        free(batch_order);
        return rc;
    }
    return ORACLE_ERR_ARG;
}

/* ------------------------------------------------------------------------------------------
 * Storage rounding (this build's bf16 store; the paper has none).
 * fp32 -> bf16 keeps the upper 16 bits, rounding to nearest, ties to even.
 * ---------------------------------------------------------------------------------------- */

uint16_t oracle_bf16_from_f32(float v) {
    uint32_t u;
    memcpy(&u, &v, 4);
    uint32_t exponent = (u >> 23) & 0xFFu;
    uint32_t mantissa = u & 0x7FFFFFu;
    if (exponent == 0xFFu && mantissa != 0) {
        /* NaN: keep sign and upper payload bits, force the quiet bit so it stays a NaN. */
        return (uint16_t)((u >> 16) | 0x0040u);
    }
    uint32_t upper = u >> 16;
    uint32_t lower = u & 0xFFFFu;
    if (lower > 0x8000u) {
        upper += 1; /* above the midpoint: round up (may carry into the exponent, up to Inf) */
    } else if (lower == 0x8000u) {
        if (upper & 1u) upper += 1; /* exactly halfway: go to the even neighbour */
    }
    return (uint16_t)upper;
}

float oracle_f32_from_bf16(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16; /* widening is exact */
    float v;
    memcpy(&v, &u, 4);
    return v;
}

void oracle_store_bf16(const float* in, int64_t count, uint16_t* out) {
    for (int64_t i = 0; i < count; ++i) out[i] = oracle_bf16_from_f32(in[i]);
}

/* ------------------------------------------------------------------------------------------
 * Standardisation (Algorithm 1, the two standardise lines): (v - mu) / sigma.
 * Two separately rounded binary32 operations; never a reciprocal multiply, never fused.
 * ---------------------------------------------------------------------------------------- */

float oracle_standardize(float v, float mu, float sigma) {
    volatile float centred = v - mu; /* volatile: one rounding here, whatever the compiler does */
    volatile float scaled = centred / sigma;
    return scaled;
}

/* ------------------------------------------------------------------------------------------
 * Index-batching (Sec. 4.1): one copy of the data and a start per window;
 * x = data[start : start+P], y = data[start+P : start+P+Q], standardised per feature.
 * ---------------------------------------------------------------------------------------- */

/* storage: 0 = fp32 series, 1 = bf16 series (uint16 bit patterns). */
static float series_at(const void* series, int storage, int64_t t, int64_t node, int64_t f,
                       int64_t N, int64_t F) {
    int64_t off = (t * N + node) * F + f;
    if (storage == 1) return oracle_f32_from_bf16(((const uint16_t*)series)[off]);
    return ((const float*)series)[off];
}

/* Builds one batch.  starts[j] is the start of sample j, j < count.
 * out_x is [count, P, N, F], out_y is [count, Q, N, F], fp32, contiguous. */
int oracle_build_batch(const void* series, int storage, int64_t T, int64_t N, int64_t F,
                       int64_t P, int64_t Q, const float* mean, const float* std,
                       const int32_t* starts, int64_t count, float* out_x, float* out_y) {
    if (!series || !mean || !std || !starts || !out_x || !out_y) return ORACLE_ERR_ARG;
    if (storage != 0 && storage != 1) return ORACLE_ERR_ARG;
    int64_t n = oracle_window_count(T, P, Q);
    for (int64_t j = 0; j < count; ++j) {
        int64_t start = starts[j];
        if (start < 0 || start >= n) return ORACLE_ERR_ARG;
        for (int64_t p = 0; p < P; ++p)
            for (int64_t node = 0; node < N; ++node)
                for (int64_t f = 0; f < F; ++f)
                    out_x[((j * P + p) * N + node) * F + f] = oracle_standardize(
                        series_at(series, storage, start + p, node, f, N, F), mean[f], std[f]);
        for (int64_t q = 0; q < Q; ++q)
            for (int64_t node = 0; node < N; ++node)
                for (int64_t f = 0; f < F; ++f)
                    out_y[((j * Q + q) * N + node) * F + f] = oracle_standardize(
                        series_at(series, storage, start + P + q, node, f, N, F), mean[f], std[f]);
    }
    return ORACLE_OK;
}

/* Same batch with bf16 outputs (this build's reduced-precision output option; the paper has
 * none): every standardised fp32 value is rounded to bf16, nearest even, as its last step. */
int oracle_build_batch_bf16_out(const void* series, int storage, int64_t T, int64_t N, int64_t F,
                                int64_t P, int64_t Q, const float* mean, const float* std,
                                const int32_t* starts, int64_t count, uint16_t* out_x,
                                uint16_t* out_y) {
    if (!series || !mean || !std || !starts || !out_x || !out_y) return ORACLE_ERR_ARG;
    if (storage != 0 && storage != 1) return ORACLE_ERR_ARG;
    int64_t n = oracle_window_count(T, P, Q);
    for (int64_t j = 0; j < count; ++j) {
        int64_t start = starts[j];
        if (start < 0 || start >= n) return ORACLE_ERR_ARG;
        for (int64_t p = 0; p < P + Q; ++p)
            for (int64_t node = 0; node < N; ++node)
                for (int64_t f = 0; f < F; ++f) {
                    float v = oracle_standardize(series_at(series, storage, start + p, node, f, N, F),
                                                 mean[f], std[f]);
                    uint16_t b = oracle_bf16_from_f32(v);
                    if (p < P) out_x[((j * P + p) * N + node) * F + f] = b;
                    else out_y[((j * Q + (p - P)) * N + node) * F + f] = b;
                }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------
 * What Algorithm 1 (the standard preprocessing) materialises: for every window w the block
 * x_all[w] = data[w .. w+P) and the block y_all[w] = data[w+P .. w+P+Q), the slice one input
 * length ahead, all blocks stacked and every element standardised.  Memory grows as Eq. 1, so
 * this is for tiny inputs: it is the brute-force definition that index-batching must reproduce
 * sample for sample.
 * x_all is [n, P, N, F], y_all is [n, Q, N, F].
 * ---------------------------------------------------------------------------------------- */
int oracle_alg1_preprocess(const float* data, int64_t T, int64_t N, int64_t F, int64_t P,
                           int64_t Q, const float* mean, const float* std, float* x_all,
                           float* y_all) {
    if (!data || !mean || !std || !x_all || !y_all) return ORACLE_ERR_ARG;
    int64_t n = oracle_window_count(T, P, Q);
    int64_t row = N * F;
    /* the append loop and the stack */
    for (int64_t window = 0; window < n; ++window) {
        memcpy(x_all + window * P * row, data + window * row, (size_t)(P * row) * sizeof(float));
        memcpy(y_all + window * Q * row, data + (window + P) * row,
               (size_t)(Q * row) * sizeof(float));
    }
    /* standardise the two stacks */
    for (int64_t e = 0; e < n * P * row; ++e)
        x_all[e] = oracle_standardize(x_all[e], mean[e % F], std[e % F]);
    for (int64_t e = 0; e < n * Q * row; ++e)
        y_all[e] = oracle_standardize(y_all[e], mean[e % F], std[e % F]);
    return ORACLE_OK;
}

/* Algorithm 1's own statistics: one scalar mean and one scalar standard deviation
 * (population, divisor = count) over every element of x_train, the first
 * round(0.70 * n) windows of the stacked x.  Elements near the ends of the training range
 * appear in fewer windows and so weigh less; features are mixed.  fp64 accumulation,
 * window-major order.  round() is round-half-to-even as in the listing's language.  The
 * listing fixes the training fraction at 0.70 and its caption allows other splits, hence the
 * parameter. */
int oracle_alg1_train_stats_fraction(const float* data, int64_t T, int64_t N, int64_t F, int64_t P,
                                     int64_t Q, double fraction, double* mean_out, double* std_out) {
    if (!data || !mean_out || !std_out) return ORACLE_ERR_ARG;
    int64_t n = oracle_window_count(T, P, Q);
    int64_t n_train = (int64_t)nearbyint((double)n * fraction);
    int64_t row = N * F;
    int64_t count = n_train * P * row;
    if (count <= 0) return ORACLE_ERR_ARG;
    double sum = 0.0;
    for (int64_t w = 0; w < n_train; ++w)
        for (int64_t e = 0; e < P * row; ++e) sum += (double)data[w * row + e];
    double mean = sum / (double)count;
    double sq = 0.0;
    for (int64_t w = 0; w < n_train; ++w)
        for (int64_t e = 0; e < P * row; ++e) {
            double d = (double)data[w * row + e] - mean;
            sq += d * d;
        }
    *mean_out = mean;
    *std_out = sqrt(sq / (double)count);
    return ORACLE_OK;
}

/* Algorithm 1 as listed: the training part is the first 70 % of the windows. */
int oracle_alg1_train_stats(const float* data, int64_t T, int64_t N, int64_t F, int64_t P,
                            int64_t Q, double* mean_out, double* std_out) {
    return oracle_alg1_train_stats_fraction(data, T, N, F, P, Q, 0.70, mean_out, std_out);
}

/* Stage 1 of the preprocessing (the data-growth figure of Sec. 3.3: time-of-day information
 * is added to the data as one more feature, the same value for every node of a timestep).
 * out[t, node, 0..F-1] = data[t, node, :], out[t, node, F] = (t mod period) / period, the
 * quotient taken in binary32 (both operands are small integers, exactly representable). */
int oracle_add_time_of_day(const float* data, int64_t T, int64_t N, int64_t F, int64_t period,
                           float* out) {
    if (!data || !out || T <= 0 || N <= 0 || F <= 0 || period <= 0 || period >= (1 << 24))
        return ORACLE_ERR_ARG;
    for (int64_t t = 0; t < T; ++t) {
        volatile float tod = (float)(t % period) / (float)period;
        for (int64_t node = 0; node < N; ++node) {
            for (int64_t f = 0; f < F; ++f)
                out[(t * N + node) * (F + 1) + f] = data[(t * N + node) * F + f];
            out[(t * N + node) * (F + 1) + F] = tod;
        }
    }
    return ORACLE_OK;
}

/* Per-feature statistics over the whole series (this build's default standardisation rule;
 * Algorithm 1's caption allows other rules): mean[f] and population standard deviation
 * std[f] of all T*N values of feature f.  fp64 throughout: each timestep row is summed
 * node by node, the row sums are summed in time order; second pass for squared deviations
 * in the same order; rounded to fp32 once at the end. */
int oracle_series_stats(const float* data, int64_t T, int64_t N, int64_t F, float* mean_out,
                        float* std_out) {
    if (!data || !mean_out || !std_out || T <= 0 || N <= 0 || F <= 0) return ORACLE_ERR_ARG;
    double count = (double)T * (double)N;
    for (int64_t f = 0; f < F; ++f) {
        double total = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double row_sum = 0.0;
            for (int64_t node = 0; node < N; ++node) row_sum += (double)data[(t * N + node) * F + f];
            total += row_sum;
        }
        double mean = total / count;
        double total_sq = 0.0;
        for (int64_t t = 0; t < T; ++t) {
            double row_sq = 0.0;
            for (int64_t node = 0; node < N; ++node) {
                double d = (double)data[(t * N + node) * F + f] - mean;
                row_sq += d * d;
            }
            total_sq += row_sq;
        }
        mean_out[f] = (float)mean;
        std_out[f] = (float)sqrt(total_sq / count);
    }
    return ORACLE_OK;
}
