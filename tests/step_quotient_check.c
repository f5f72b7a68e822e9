/* Host check of the division sequence that the quantised epilogue uses for t / step (one divisor, many
 * dividends): y = RN(1/step), q0 = RN(t y), r = fma(-step, q0, t), q1 = fma(r, y, q0) must equal the IEEE
 * quotient RN(t / step).  Exhaustive over every dividend whose quotient lies in [2^-2, 2^10) (the range in
 * which the rounded integer code depends on the quotient's last bit), for the divisors given on the command
 * line and for a pseudo-random set (those with a stride over the dividends).
 * Prints one line per divisor with the number of dividends and of mismatches; exit status 1 on any mismatch.
 * Build: gcc -O2 -ffp-contract=off -o step_quotient_check step_quotient_check.c -lm */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static uint32_t bits_of(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float float_of(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

static int fast_ok(float step) {
    const uint32_t b = bits_of(step), e = (b >> 23) & 0xFFu;
    return e >= 64u && e <= 190u && (b & 0x7FFFFFu) != 0x7FFFFFu;
}

static long check(float step, uint32_t stride, long* count) {
    volatile float y = 1.0f / step;
    const uint32_t lo = bits_of(step * 0.25f), hi = bits_of(step * 1024.0f);
    long bad = 0, n = 0;
    for (uint32_t u = lo; u < hi; u += stride) {
        for (int sign = 0; sign < 2; ++sign) {
            const float t = float_of(u | ((uint32_t)sign << 31));
            volatile float q0 = t * y;
            const float r = fmaf(-step, q0, t);
            const float q1 = fmaf(r, y, q0);
            const float want = t / step;
            if (bits_of(q1) != bits_of(want)) {
                if (bad < 5) fprintf(stderr, "step %a t %a: %a != %a\n", step, t, q1, want);
                ++bad;
            }
            ++n;
        }
    }
    *count = n;
    return bad;
}

int main(int argc, char** argv) {
    long total_bad = 0;
    for (int i = 1; i < argc; ++i) {
        const float step = strtof(argv[i], NULL);
        if (!fast_ok(step)) { printf("step %a skipped (the sequence is not used for it)\n", step); continue; }
        long n, bad = check(step, 1, &n);
        printf("step %a: %ld dividends, %ld mismatches\n", step, n, bad);
        total_bad += bad;
    }
    uint32_t s = 12345u;
    for (int i = 0; i < 64; ++i) {
        s = s * 1664525u + 1013904223u;
        /* significand from the generator, exponent 2^-10 .. 2^5 */
        const float step = float_of(((117u + (s >> 28)) << 23) | (s & 0x7FFFFFu));
        if (!fast_ok(step)) continue;
        long n, bad = check(step, 61, &n);
        if (bad) printf("step %a: %ld dividends, %ld mismatches\n", step, n, bad);
        total_bad += bad;
    }
    printf("total mismatches %ld\n", total_bad);
    return total_bad ? 1 : 0;
}
