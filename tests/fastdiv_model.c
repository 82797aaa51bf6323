/*
 * CPU model of the division the gather kernel uses on its fast path, checked against the
 * correctly rounded IEEE binary32 division of the host.  Not the oracle and not the kernel:
 * a stand-alone proof harness for one arithmetic identity.
 *
 * Claim: for sigma finite with biased exponent in [95, 159] (|sigma| in [2^-32, 2^32)) and r =
 * binary32(1.0 / (double)sigma), compute for ANY binary32 d
 *     q0 = d*r;  e0 = fma(-sigma, q0, d);  q1 = fma(e0, r, q0);
 *     e1 = fma(-sigma, q1, d);  q = fma(e1, r, q1).
 * If q's biased exponent lies in [96, 158] then q equals RN(d / sigma) bit for bit (Markstein's
 * correction step applied to a faithful quotient with a correctly rounded reciprocal; a quotient
 * of that size implies a dividend for which nothing overflowed or underflowed); otherwise the
 * caller divides the ordinary way.  The check below applies exactly that rule, so it covers the
 * acceptance test as well as the arithmetic: zeros, subnormals, infinities and NaNs included.
 *
 * usage: fastdiv_model <mode> ...
 *   exhaustive <sigma_bits_hex>            every one of the 2^32 dividends
 *   random <n_sigma> <stride> <seed>       n random sigmas x every stride-th dividend
 * prints "bad=<count>" and exits non-zero if any quotient differs.
 * Build: gcc -O2 -mfma -ffp-contract=off -fopenmp.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static inline float asf(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t asu(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

static inline int quotient_accepted(float q) {
    return ((asu(q) & 0x7FFFFFFFu) - (96u << 23)) < (63u << 23); /* biased exponent in [96, 158] */
}

static inline float fast_divide(float d, float sigma, float r) {
    float q0 = d * r;
    float e0 = fmaf(-sigma, q0, d);
    float q1 = fmaf(e0, r, q0);
    float e1 = fmaf(-sigma, q1, d);
    return fmaf(e1, r, q1);
}

static uint64_t check_sigma(uint32_t sigma_bits, uint64_t stride, uint64_t offset) {
    const float sigma = asf(sigma_bits);
    const float r = (float)(1.0 / (double)sigma);
    uint64_t bad = 0;
#pragma omp parallel for reduction(+ : bad) schedule(dynamic, 65536)
    for (uint64_t u = offset; u < (1ull << 32); u += stride) {
        const float d = asf((uint32_t)u);
        const float fast = fast_divide(d, sigma, r);
        const float got = quotient_accepted(fast) ? fast : d / sigma; /* the kernel's rule */
        const float want = d / sigma;
        if (asu(want) != asu(got) && !(want != want && got != got)) bad++;
    }
    return bad;
}

static uint64_t splitmix(uint64_t* s) {
    uint64_t z = (*s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

int main(int argc, char** argv) {
    uint64_t bad = 0;
    if (argc >= 3 && strcmp(argv[1], "exhaustive") == 0) {
        bad = check_sigma((uint32_t)strtoul(argv[2], 0, 16), 1, 0);
    } else if (argc >= 5 && strcmp(argv[1], "random") == 0) {
        uint64_t n = strtoull(argv[2], 0, 10), stride = strtoull(argv[3], 0, 10), seed = strtoull(argv[4], 0, 10);
        for (uint64_t k = 0; k < n; ++k) {
            uint64_t h = splitmix(&seed);
            uint32_t expo = 95u + (uint32_t)((h >> 40) % 65u);          /* biased exponent 95..159 */
            uint32_t bits = ((uint32_t)(h >> 63) << 31) | (expo << 23) | ((uint32_t)h & 0x7FFFFFu);
            bad += check_sigma(bits, stride, splitmix(&seed) % stride);
        }
    } else {
        fprintf(stderr, "usage: %s exhaustive <hex> | random <n> <stride> <seed>\n", argv[0]);
        return 2;
    }
    printf("bad=%llu\n", (unsigned long long)bad);
    return bad ? 1 : 0;
}
