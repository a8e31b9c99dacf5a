/* Check of the division the large-tensor activation quantizer uses for u = amax / (6 S):
 *   r = RN(1 / b);  q0 = RN(a * r);  q = fma(fma(-q0, b, a), r, q0)
 * against the correctly rounded quotient RN(a / b), for operands whose magnitudes stay well inside the
 * normal range (the kernel's host side admits only such S).  Structured sweep: every b from a set of
 * mantissas that stresses the reciprocal's rounding (all 2^11 leading patterns, runs of ones and zeros,
 * the neighbours of powers of two), against a values on the bf16 grid (what amax of a bf16 tensor is)
 * and pseudo-random full-precision ones, over a range of exponent differences.
 * Prints the number of mismatches; exit status 0 iff none.  Compile: gcc -O2 -ffp-contract=off -lm. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

static float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

static long check(float a, float b)
{
    volatile float r = 1.0f / b;
    volatile float q0 = a * r;
    volatile float res = fmaf(-q0, b, a);
    volatile float q = fmaf(res, r, q0);
    volatile float want = a / b;
    return f2u(q) != f2u(want);
}

int main(void)
{
    long bad = 0, total = 0;
    uint64_t s = 88172645463325252ULL;
    for (uint32_t hi = 0; hi < 2048; ++hi) {
        const uint32_t tails[6] = {0u, 1u, 0xFFFu, 0xFFEu, 0x800u, 0x555u};
        for (int t = 0; t < 6; ++t) {
            const uint32_t mb = (hi << 12) | tails[t];
            for (int eb = -20; eb <= 20; eb += 8) {
                const float b = u2f(((uint32_t)(127 + eb) << 23) | mb);
                for (int k = 0; k < 48; ++k) {
                    s ^= s << 13; s ^= s >> 7; s ^= s << 17;
                    uint32_t ma = (uint32_t)(s & 0x7FFFFF);
                    if (k & 1) ma &= 0x7F0000;                       /* bf16 grid */
                    if ((k & 7) == 2) ma = 0x7FFFFF - (uint32_t)((s >> 30) & 15);
                    if ((k & 7) == 4) ma = (uint32_t)((s >> 30) & 15);
                    const int ea = eb + (int)((s >> 40) % 41) - 20;
                    const float a = u2f(((uint32_t)(127 + ea) << 23) | ma);
                    bad += check(a, b);
                    ++total;
                }
            }
        }
    }
    printf("%ld mismatches of %ld\n", bad, total);
    return bad != 0;
}
