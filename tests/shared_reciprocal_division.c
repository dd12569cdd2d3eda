/*
 * Check of the division used by the fused kernel for unsplit items: for a count
 * k (1..64) and a binary32 numerator a,
 *     y = RN(1/k);  q0 = RN(a*y);  r = fma(-k, q0, a);  q = fma(r, y, q0);
 *     if q is neither a normal number nor zero:  q = a / k
 * must give the bits of a / k.  The only exception is a = -0 (the sequence gives
 * +0), which cannot occur in the kernel: its sums start from +0.
 *
 *   shared_reciprocal_division <k_first> <k_last> <stride>
 * walks the numerators' bit patterns 0, stride, 2*stride, ... and prints the
 * number of mismatches (NaN against NaN counts as a match); exit status 1 if
 * there is any.  stride 1 is the complete check (about 15 s per count on 8
 * cores); the test suite runs a strided pass over all counts.
 * Build: gcc -O2 -mfma -ffp-contract=off -fopenmp (fmaf must be a fused operation).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static inline float as_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static inline uint32_t as_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

int main(int argc, char **argv)
{
    const int k0 = argc > 1 ? atoi(argv[1]) : 1, k1 = argc > 2 ? atoi(argv[2]) : 64;
    const long long stride = argc > 3 ? atoll(argv[3]) : 1;
    if (k0 < 1 || k1 > 64 || stride < 1) return 2;
    unsigned long long bad_total = 0;
    for (int k = k0; k <= k1; ++k) {
        volatile float kv = (float)k;            /* keeps the compiler from folding the divisions */
        const float kf = kv;
        const float y = 1.0f / kf;
        unsigned long long bad = 0;
#pragma omp parallel for reduction(+ : bad) schedule(static)
        for (long long i = 0; i < (1LL << 32); i += stride) {
            const float a = as_float((uint32_t)i);
            if ((uint32_t)i == 0x80000000u) continue;              /* -0: see above */
            const float want = a / kf;
            const float q0 = a * y;
            const float r = fmaf(-kf, q0, a);
            float q = fmaf(r, y, q0);
            if (!(isnormal(q) || q == 0.0f)) q = a / kf;
            if (as_bits(q) != as_bits(want) && !(q != q && want != want)) ++bad;
        }
        if (bad) printf("k=%d: %llu mismatches\n", k, bad);
        bad_total += bad;
    }
    printf("mismatches: %llu\n", bad_total);
    return bad_total ? 1 : 0;
}
