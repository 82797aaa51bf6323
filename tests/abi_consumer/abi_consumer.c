/* A consumer of the C ABI written in plain C: no Python, no torch, only pgti.h and the HIP runtime for
 * device buffers and a stream.  It loads a small synthetic series, generates one rank's share of an
 * epoch, builds the first and the last batch on a stream of its own and writes the share and the
 * batches to a file; tests/test_abi_consumer.py checks that file against the CPU oracle.
 *
 * usage: abi_consumer <out file> <T> <N> <F> <P> <Q> <B> <seed> <epoch> <rank> <world> <bf16 storage 0|1>
 * The series is value(t, n, f) = ((t * 131 + n * 17 + f * 7) mod 1009) * 0.125 - 40.0 (exact in fp32),
 * standardised with mean[f] = 20 + f, std[f] = 7.5 + 0.25 f.
 * File layout (native endian): int64 n_share, int64 nb, int32 first_count, int32 last_count,
 * int32 share[n_share], float x0[B*P*N*F], float y0[B*Q*N*F], float x_last[...], float y_last[...]. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "pgti.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at line %d\n", (int)e_, __LINE__); return 3; } } while (0)
#define PGTI_OK_(x) do { long long r_ = (long long)(x); if (r_ < 0) { fprintf(stderr, "pgti error %lld at line %d: %s\n", r_, __LINE__, pgti_last_error()); return 4; } } while (0)

int main(int argc, char** argv) {
    if (argc != 13) { fprintf(stderr, "usage: see the source\n"); return 2; }
    const char* out_path = argv[1];
    const long long T = atoll(argv[2]);
    const int N = atoi(argv[3]), F = atoi(argv[4]), P = atoi(argv[5]), Q = atoi(argv[6]), B = atoi(argv[7]);
    const unsigned long long seed = strtoull(argv[8], 0, 10), epoch = strtoull(argv[9], 0, 10);
    const unsigned rank = (unsigned)atoi(argv[10]), world = (unsigned)atoi(argv[11]);
    const int bf16 = atoi(argv[12]);

    const size_t elems = (size_t)T * N * F;
    float* series = (float*)malloc(elems * sizeof(float));
    float* mean = (float*)malloc(F * sizeof(float));
    float* std = (float*)malloc(F * sizeof(float));
    if (!series || !mean || !std) return 5;
    for (long long t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n)
            for (int f = 0; f < F; ++f)
                series[((size_t)t * N + n) * F + f] = (float)((t * 131 + n * 17 + f * 7) % 1009) * 0.125f - 40.0f;
    for (int f = 0; f < F; ++f) { mean[f] = 20.0f + (float)f; std[f] = 7.5f + 0.25f * (float)f; }

    pgti_ctx* ctx = 0;
    PGTI_OK_(pgti_create(&ctx, 0));
    PGTI_OK_(pgti_load_series(ctx, series, T, N, F, P, Q, B, bf16 ? PGTI_BF16 : PGTI_F32, mean, std));
    int64_t n_share = 0;
    PGTI_OK_(pgti_epoch_indices(ctx, seed, epoch, rank, world, &n_share));
    const int64_t nb = pgti_num_batches(ctx);
    PGTI_OK_(nb);
    int32_t* share = (int32_t*)malloc((size_t)(n_share > 0 ? n_share : 1) * sizeof(int32_t));
    PGTI_OK_(pgti_get_indices(ctx, share, n_share));

    const size_t xe = (size_t)B * P * N * F, ye = (size_t)B * Q * N * F;
    float *dx[2], *dy[2];
    hipStream_t stream;
    HIP_OK(hipSetDevice(0));
    HIP_OK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking));
    for (int k = 0; k < 2; ++k) {
        HIP_OK(hipMalloc((void**)&dx[k], xe * sizeof(float)));
        HIP_OK(hipMalloc((void**)&dy[k], ye * sizeof(float)));
        HIP_OK(hipMemsetAsync(dx[k], 0, xe * sizeof(float), stream));
        HIP_OK(hipMemsetAsync(dy[k], 0, ye * sizeof(float), stream));
    }
    const int first_count = pgti_build_batch(ctx, 0, dx[0], dy[0], stream);
    PGTI_OK_(first_count);
    const int last_count = pgti_build_batch(ctx, nb - 1, dx[1], dy[1], stream);
    PGTI_OK_(last_count);
    float* hx = (float*)malloc(xe * sizeof(float));
    float* hy = (float*)malloc(ye * sizeof(float));
    FILE* out = fopen(out_path, "wb");
    if (!out || !hx || !hy) return 6;
    const int64_t head[2] = {n_share, nb};
    const int32_t counts[2] = {first_count, last_count};
    fwrite(head, sizeof(head), 1, out);
    fwrite(counts, sizeof(counts), 1, out);
    fwrite(share, sizeof(int32_t), (size_t)n_share, out);
    for (int k = 0; k < 2; ++k) {
        HIP_OK(hipMemcpyAsync(hx, dx[k], xe * sizeof(float), hipMemcpyDeviceToHost, stream));
        HIP_OK(hipMemcpyAsync(hy, dy[k], ye * sizeof(float), hipMemcpyDeviceToHost, stream));
        HIP_OK(hipStreamSynchronize(stream));
        fwrite(hx, sizeof(float), xe, out);
        fwrite(hy, sizeof(float), ye, out);
    }
    fclose(out);
    /* an error path through the same boundary */
    if (pgti_build_batch(ctx, nb, dx[0], dy[0], stream) != PGTI_ERR_RANGE) { fprintf(stderr, "expected PGTI_ERR_RANGE\n"); return 7; }
    pgti_destroy(ctx);
    for (int k = 0; k < 2; ++k) { HIP_OK(hipFree(dx[k])); HIP_OK(hipFree(dy[k])); }
    HIP_OK(hipStreamDestroy(stream));
    free(series); free(mean); free(std); free(share); free(hx); free(hy);
    printf("abi_consumer ok: n_share=%lld nb=%lld first=%d last=%d\n", (long long)n_share, (long long)nb, first_count, last_count);
    return 0;
}
