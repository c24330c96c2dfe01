/* Exhaustive check, on the CPU, of the quotient filter of the quantizer kernel
 * (paper_2306_00978_amd/csrc/awq_quantize.hip, fast_rint_quotient).
 *
 * The codes of the quantizer (Sec. 3.2, Eq. 1 in its asymmetric form) are rint(fl(n / d)) with fl the
 * correctly rounded binary32 division and d the group's step, a positive normal binary16 value.
 * The kernel forms q0 = fl(n * r), r = fma(fma(-d, r0, 1), r0, r0), r0 the hardware reciprocal of
 * d (within one ulp of 1/d), and keeps rint(q0) unless q0 lies within BAND = 2^-16 of a
 * half-integer (|q0 - rint(q0)| > 1/2 - BAND), in which case it divides properly.  Claim checked here: for EVERY step d, every r0
 * within one ulp of the correctly rounded reciprocal, every half-integer h = k + 1/2 with
 * |h| < 34 and every binary32 numerator within WINDOW ulps of h * d (the only numerators whose
 * rounding can be in doubt, plus a margin), whenever q0 is outside the band, rint(q0) equals
 * rint(fl(n / d)); and for numerators spread over the whole range |n / d| < 32 the distance
 * |q0 - fl(n / d)| stays below 2^-17, half the band.  Exit status 0 = the claim holds.
 *
 * Build: gcc -O2 -ffp-contract=off -o quotient_filter_check quotient_filter_check.c -lm */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

static float f16_bits_to_float(uint16_t h)
{
    const int e = (h >> 10) & 31, m = h & 1023;
    return ldexpf((float)(1024 + m), e - 25);          /* normal values only */
}

static float refined(float d, float r0) { return fmaf(fmaf(-d, r0, 1.0f), r0, r0); }

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rng(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 7;
    rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}

int main(void)
{
#ifndef BAND_VALUE
#define BAND_VALUE 1.52587890625e-05f                   /* 2^-16, as in the kernel */
#endif
    const float BAND = BAND_VALUE;
    const int WINDOW = 12;
    long long checked = 0, in_band = 0, bad = 0, spread = 0;
    double worst = 0.0;
    for (int e = 1; e <= 30; ++e)
        for (int m = 0; m < 1024; ++m) {
            const float d = f16_bits_to_float((uint16_t)((e << 10) | m));
            const float rn = 1.0f / d;
            const float cand[3] = {rn, nextafterf(rn, INFINITY), nextafterf(rn, 0.0f)};
            for (int c = 0; c < 3; ++c) {
                const float r = refined(d, cand[c]);
                for (int k = -34; k <= 33; ++k) {
                    const float h = (float)k + 0.5f;
                    float n = h * d;                     /* a numerator next to the tie */
                    for (int w = 0; w < WINDOW; ++w) n = nextafterf(n, -INFINITY);
                    for (int w = -WINDOW; w <= WINDOW; ++w, n = nextafterf(n, INFINITY)) {
                        const float q0 = n * r, qe = n / d;
                        const float off = fabsf(q0 - rintf(q0));        /* exact; what the kernel tracks */
                        ++checked;
                        if (off > 0.5f - BAND) { ++in_band; continue; } /* the kernel divides properly */
                        if (fabsf(q0) < 32.0f && rintf(q0) != rintf(qe)) {
                            if (bad++ < 10)
                                printf("MISS d=%a r0=%a n=%a q0=%a qe=%a\n", d, cand[c], n, q0, qe);
                        }
                    }
                }
                /* numerators anywhere in the range the codes depend on */
                for (int t = 0; t < 24; ++t) {
                    const float u = (float)(rng() >> 8) * (1.0f / 16777216.0f);      /* [0,1) */
                    const float n = (u * 64.0f - 32.0f) * d;
                    const float q0 = n * r, qe = n / d;
                    if (fabsf(q0) >= 32.0f) continue;
                    const double diff = fabs((double)q0 - (double)qe);
                    if (diff > worst) worst = diff;
                    ++spread;
                    if (diff >= 7.62939453125e-06) {                                   /* 2^-17 */
                        if (bad++ < 10) printf("FAR d=%a r0=%a n=%a q0=%a qe=%a\n", d, cand[c], n, q0, qe);
                    }
                }
            }
        }
    printf("near-tie numerators checked %lld (in band %lld), spread numerators %lld, "
           "largest |q0 - fl(n/d)| %.3g, misses %lld\n", checked, in_band, spread, worst, bad);
    return bad ? 1 : 0;
}
