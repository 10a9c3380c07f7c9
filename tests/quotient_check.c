/* Host check of the arithmetic claim behind the kernels' quantiser: the IEEE
 * quotient x / s equals  q2  with
 *     y  = RN(1 / s)          (one division per scale)
 *     q0 = RN(x * y)
 *     q1 = RN(q0 + RN(x - s * q0) * y)      (remainder exact: fused multiply-add)
 *     q2 = RN(q1 + RN(x - s * q1) * y)
 * whenever nothing under- or overflows.  This file restates that claim for the
 * CPU (it shares no code with the kernels or with the oracle) and tests it
 *   (a) exhaustively over all 2^23 significands of x for a set of scales that
 *       includes the significands closest to 1 and to 2, and
 *   (b) on random pairs with quotients across the INT4 / INT8 code ranges.
 * Prints "mismatches <n>"; exit status 1 if n > 0.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }

static float corrected(float x, float s, float y)
{
    float q = x * y;
    q = fmaf(fmaf(-s, q, x), y, q);
    q = fmaf(fmaf(-s, q, x), y, q);
    return q;
}

int main(int argc, char **argv)
{
    const int n_scales = argc > 1 ? atoi(argv[1]) : 96;
    const long n_random = argc > 2 ? atol(argv[2]) : 50000000L;
    long bad = 0;
    for (int k = 0; k < n_scales; ++k) {
        uint64_t r = 0x9E3779B97F4A7C15ull * (uint64_t)(k + 1);
        r ^= r >> 29; r *= 0xBF58476D1CE4E5B9ull; r ^= r >> 32;
        uint32_t sm = (uint32_t)r & 0x7fffffu;
        if (k < 32) sm = (uint32_t)k;                        /* significands just above 1 */
        else if (k < 64) sm = 0x7fffffu - (uint32_t)(k - 32); /* ... just below 2 */
        const float s = from_bits((110u << 23) | sm);
        const float y = 1.0f / s;
        for (uint32_t xm = 0; xm < (1u << 23); ++xm) {
            const float x = from_bits((112u << 23) | xm);
            bad += corrected(x, s, y) != x / s;
        }
    }
    uint64_t g = 88172645463325252ull;
    for (long i = 0; i < n_random; ++i) {
        g ^= g << 13; g ^= g >> 7; g ^= g << 17;
        const uint32_t sm = (uint32_t)g & 0x7fffffu;
        const int se = 100 + (int)((g >> 23) % 41); /* scales 2^-27 .. 2^13 */
        float s = from_bits(((uint32_t)se << 23) | sm);
        if (s < 1e-8f) s = 1e-8f;
        const int qe = -3 + (int)((g >> 55) % 12); /* quotients about 2^-3 .. 2^9 */
        const float x = from_bits(((uint32_t)(se + qe) << 23) | ((uint32_t)(g >> 32) & 0x7fffffu) | ((uint32_t)(g >> 63) << 31));
        const float y = 1.0f / s;
        bad += corrected(x, s, y) != x / s;
    }
    printf("mismatches %ld\n", bad);
    return bad != 0;
}
