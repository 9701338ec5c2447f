/*
 * Exhaustive pin of the oracle's fp32 -> fp16 and fp32 -> bf16 round-to-nearest-even
 * casts over all 2^32 inputs.
 *
 *   fp16: against the CPU's hardware converter (F16C vcvtps2ph), an independent
 *         implementation of IEEE-754 round-to-nearest-even narrowing.
 *   bf16: against a compare-the-two-neighbours formulation evaluated in double:
 *         truncate toward zero, form the next value away from zero, pick the
 *         nearer one, and on an exact tie the one whose last bit is zero.  The
 *         overflow threshold is treated as if the exponent range were unbounded
 *         (2^128 stands for the value after the largest finite one).
 *
 * Prints "mismatches_f16=<n> mismatches_bf16=<n>" and exits 0 iff both are 0.
 * Built by tests/test_oracle_casts.py together with oracle/zi_oracle.c.
 */
#include <immintrin.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/zi_oracle.h"

static inline float bf(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }

static uint16_t bf16_by_neighbours(uint32_t bits)
{
    const uint32_t a = bits & 0x7FFFFFFFu;
    const uint16_t sign = (uint16_t)(bits >> 31 << 15);
    if (a > 0x7F800000u) return 0xFFFFu;           /* NaN: caller only checks NaN-ness */
    if (a == 0x7F800000u) return (uint16_t)(sign | 0x7F80u);
    const uint32_t lo = a & 0xFFFF0000u;
    const uint32_t hi = lo + 0x10000u;
    const double x = (double)bf(a);
    const double lov = (double)bf(lo);
    const double hiv = (hi >= 0x7F800000u) ? ldexp(1.0, 128) : (double)bf(hi);
    const double dl = x - lov, dh = hiv - x;       /* exact: all three are doubles with few bits */
    uint32_t pick;
    if (dl < dh) pick = lo;
    else if (dh < dl) pick = hi;
    else pick = ((lo >> 16) & 1u) ? hi : lo;
    return (uint16_t)(sign | (pick >> 16));
}

int main(int argc, char** argv)
{
    uint64_t stride = 1;
    if (argc > 1) stride = strtoull(argv[1], 0, 10);
    if (stride == 0) stride = 1;
    long long bad16 = 0, badbf = 0;
#pragma omp parallel for reduction(+ : bad16, badbf) schedule(static)
    for (int64_t blk = 0; blk < 65536; ++blk) {
        for (uint64_t lowbits = 0; lowbits < 65536; lowbits += stride) {
            const uint32_t bits = (uint32_t)((uint64_t)blk << 16 | lowbits);
            const float x = bf(bits);
            const int isnan_x = (bits & 0x7FFFFFFFu) > 0x7F800000u;

            const uint16_t o16 = zio_f32_to_f16(x);
            const uint16_t h16 = (uint16_t)_cvtss_sh(x, _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
            if (isnan_x) {
                if (!((o16 & 0x7C00u) == 0x7C00u && (o16 & 0x3FFu))) ++bad16;
            } else if (o16 != h16) {
                ++bad16;
            }

            const uint16_t ob = zio_f32_to_bf16(x);
            const uint16_t nb = bf16_by_neighbours(bits);
            if (isnan_x) {
                if (!((ob & 0x7F80u) == 0x7F80u && (ob & 0x7Fu))) ++badbf;
            } else if (ob != nb) {
                ++badbf;
            }
        }
    }
    printf("mismatches_f16=%lld mismatches_bf16=%lld\n", bad16, badbf);
    return (bad16 == 0 && badbf == 0) ? 0 : 1;
}
