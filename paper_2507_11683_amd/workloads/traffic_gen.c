/*
 * Seeded synthetic traffic-shaped series: the input generator shared by the tests, the smoke
 * check and the benchmark.  It stands in for the paper's traffic datasets (same shapes as
 * Table 1) and holds none of the method's arithmetic: no windows, no standardisation, no
 * shuffle.  Counter based: every value is a pure function of (data_seed, t, node), so the
 * series can be generated in any order and by any number of threads with identical bits.
 *
 *   speed[t,n] = clip( weekly(t) * (60 + A_n * sin(2*pi*t/288 + phi_n)) + 3*z(t,n), 0, 80 ),
 *                then set to 0 with probability ~1% (sensor dropout)
 *   tod[t,n]   = (t mod 288) / 288                                   (time of day)
 * laid out [T, N, 2] fp32 with the feature fastest.
 *
 * Build: gcc -O2 -fopenmp -shared -fPIC.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

/* 64-bit finaliser of MurmurHash3 (public domain, Appleby): a bijective bit mixer. */
static inline uint64_t fmix64(uint64_t k) {
    k ^= k >> 33;
    k *= UINT64_C(0xff51afd7ed558ccd);
    k ^= k >> 33;
    k *= UINT64_C(0xc4ceb9fe1a85ec53);
    k ^= k >> 33;
    return k;
}

static inline uint64_t hash3(uint64_t seed, uint64_t stream, uint64_t a, uint64_t b) {
    uint64_t h = fmix64(seed * UINT64_C(0x100000001b3) + stream);
    h = fmix64(h ^ (a + UINT64_C(0x632be59bd9b4e019)));
    return fmix64(h ^ (b + UINT64_C(0x2545f4914f6cdd1d)));
}

static inline double unit24(uint64_t bits24) { return (double)bits24 * (1.0 / 16777216.0); }

/*
 * flags bit 0: per-node amplitude A_n ~ U(4,12) and phase phi_n ~ U(0,2*pi) (else A=8, phi=0)
 * flags bit 1: weekly modulation 0.9 + 0.1*sin(2*pi*t/2016) of the deterministic part
 * out: [T, N, 2] fp32.  t_begin/t_end select a range of timesteps (rows written at their
 * absolute position in `out`), so large series can be produced in slabs.
 */
int traffic_series_fill(float* out, int64_t T, int64_t N, uint64_t data_seed, int flags,
                        int64_t t_begin, int64_t t_end) {
    const double two_pi = 6.283185307179586476925286766559;
    if (!out || T <= 0 || N <= 0) return -1;
    if (t_begin < 0) t_begin = 0;
    if (t_end > T) t_end = T;
    /* per-node amplitude and phase, as sin/cos of the phase */
    float* node_tab = (float*)malloc((size_t)N * 3 * sizeof(float));
    if (!node_tab) return -2;
    for (int64_t n = 0; n < N; ++n) {
        float amp = 8.0f, sin_p = 0.0f, cos_p = 1.0f;
        if (flags & 1) {
            uint64_t hn = hash3(data_seed, 1, (uint64_t)n, 0);
            amp = (float)(4.0 + 8.0 * unit24(hn >> 40));
            double phi = two_pi * unit24((hn >> 16) & 0xFFFFFF);
            sin_p = (float)sin(phi);
            cos_p = (float)cos(phi);
        }
        node_tab[3 * n + 0] = amp;
        node_tab[3 * n + 1] = sin_p;
        node_tab[3 * n + 2] = cos_p;
    }
#pragma omp parallel for schedule(static)
    for (int64_t t = t_begin; t < t_end; ++t) {
        double ang = two_pi * (double)(t % 288) / 288.0;
        float sin_t = (float)sin(ang), cos_t = (float)cos(ang);
        float weekly = (flags & 2) ? (float)(0.9 + 0.1 * sin(two_pi * (double)(t % 2016) / 2016.0)) : 1.0f;
        float tod = (float)(t % 288) / 288.0f;
        float* row = out + t * N * 2;
        for (int64_t n = 0; n < N; ++n) {
            float amp = node_tab[3 * n + 0], sin_p = node_tab[3 * n + 1], cos_p = node_tab[3 * n + 2];
            /* sin(a + phi) by the addition theorem: one sincos per timestep, not per value */
            float base = weekly * (60.0f + amp * (sin_t * cos_p + cos_t * sin_p));
            uint64_t h = hash3(data_seed, 2, (uint64_t)t, (uint64_t)n);
            float u1 = (float)(((h >> 40) + 1) * (1.0 / 16777216.0)); /* (0,1] */
            float u2 = (float)unit24((h >> 16) & 0xFFFFFF);
            float z = sqrtf(-2.0f * logf(u1)) * cosf((float)two_pi * u2); /* Box-Muller */
            float v = base + 3.0f * z;
            v = v < 0.0f ? 0.0f : (v > 80.0f ? 80.0f : v);
            if ((h & 0xFFFF) < 655) v = 0.0f; /* 655/65536 ~ 1% dropout */
            row[2 * n + 0] = v;
            row[2 * n + 1] = tod;
        }
    }
    free(node_tab);
    return 0;
}
