/*
 * Two identities the quantize-and-write kernel relies on, checked on the CPU in IEEE binary32 arithmetic
 * (compile with -ffp-contract=off so that only the fmaf calls fuse).
 *
 * (1) Division by qmax = 255 or 15, correctly rounded, without a division:
 *         c = RN(1 / qmax);  q0 = r * c;  q1 = fmaf(fmaf(-qmax, q0, r), c, q0)   ==   r / qmax
 *     for binary32 r in [0, 131008] (the range of max - min of two fp16 numbers).
 *     Usage: quantizer_divisions div <stride>: every stride-th binary32 number of that interval, and every
 *     r that is itself an fp16 number.  stride 1 is the exhaustive run (a minute on eight cores).
 *
 * (2) The reciprocal of an fp16 scale, correctly rounded, from any approximation within one ulp:
 *         y1 = fmaf(fmaf(-s, y0, 1), y0, y0)   ==   1 / s
 *     for every fp16 s in [2^-14, 65504] and y0 in {RN(1/s) - 1 ulp, RN(1/s), RN(1/s) + 1 ulp}, which covers
 *     every result a reciprocal instruction with an error of at most one ulp can return.
 *     Usage: quantizer_divisions rcp
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }
static uint32_t to_bits(float x) { uint32_t b; memcpy(&b, &x, 4); return b; }

static float half_to_float(uint16_t h)       /* normal and subnormal, positive */
{
    const int e = (h >> 10) & 31, m = h & 1023;
    return e == 0 ? ldexpf((float)m, -24) : ldexpf((float)(m | 1024), e - 25);
}

static int div_ok(float r, float qmax, float c)
{
    const float q0 = r * c;
    const float q1 = fmaf(fmaf(-qmax, q0, r), c, q0);
    return q1 == r / qmax;
}

int main(int argc, char **argv)
{
    if (argc >= 2 && !strcmp(argv[1], "div")) {
        const long stride = argc >= 3 ? atol(argv[2]) : 1;
        if (stride < 1) return 2;
        const float qs[2] = {255.0f, 15.0f};
        long bad = 0, n = 0;
        for (int k = 0; k < 2; ++k) {
            const float qmax = qs[k], c = 1.0f / qmax;
            const long top = (long)to_bits(131008.0f);
            long bad_k = 0, n_k = 0;
#pragma omp parallel for reduction(+ : bad_k, n_k) schedule(static)
            for (long b = 0; b <= top; b += stride) {
                bad_k += !div_ok(from_bits((uint32_t)b), qmax, c);
                ++n_k;
            }
            for (uint32_t h = 0; h < 0x7C00u; ++h) {
                bad_k += !div_ok(half_to_float((uint16_t)h), qmax, c);
                bad_k += !div_ok(2.0f * half_to_float((uint16_t)h), qmax, c);
                n_k += 2;
            }
            bad += bad_k;
            n += n_k;
        }
        printf("div: %ld values, %ld mismatches\n", n, bad);
        return bad != 0;
    }
    if (argc >= 2 && !strcmp(argv[1], "rcp")) {
        long bad = 0, n = 0;
        for (uint32_t h = 0x0400u; h < 0x7C00u; ++h) {
            const float s = half_to_float((uint16_t)h), want = 1.0f / s;
            for (int d = -1; d <= 1; ++d) {
                const float y0 = from_bits(to_bits(want) + (uint32_t)d);
                const float y1 = fmaf(fmaf(-s, y0, 1.0f), y0, y0);
                bad += y1 != want;
                ++n;
            }
        }
        printf("rcp: %ld cases, %ld mismatches\n", n, bad);
        return bad != 0;
    }
    fprintf(stderr, "usage: %s div <stride> | rcp\n", argv[0]);
    return 2;
}
