/* Host check of an arithmetic identity the quantiser kernel relies on (not part of the oracle, and no
 * code of the kernel): for a binary16 weight w and a positive binary16 or bfloat16 scale s with
 * |w| <= s * (2^bits - 1) / 2,
 *     clamp(rint(fl32(w / s)))  ==  clamp(rint(fma(fma(-x0, s, w), rs, x0))),  x0 = fl32(w * rs), rs = fl32(1 / s),
 * i.e. Appendix A's q = int(w / s) with the quotient in IEEE binary32 can be formed from one reciprocal per
 * group and two fused multiply-adds per weight.  Walks every `stride`-th finite scale (argv[1], default 1 =
 * all of them) and every non-negative binary16 numerator in range; prints one line per (format, bits) and
 * returns the number of formats with a mismatch.  Build: gcc -O2 -ffp-contract=off encode_identity_check.c -lm */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float half_to_float(uint16_t h) {
    const uint32_t e = (h >> 10) & 31u, m = h & 1023u;
    const float v = e == 0 ? ldexpf((float)m, -24) : ldexpf((float)(m + 1024u), (int)e - 25);
    return (h & 0x8000u) ? -v : v;
}
static float bfloat_to_float(uint16_t b) {
    const uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

int main(int argc, char** argv) {
    const int stride = argc > 1 ? atoi(argv[1]) : 1;
    static float W[0x7c00];
    int failed = 0;
    if (stride < 1) return 99;
    for (int i = 0; i < 0x7c00; ++i) W[i] = half_to_float((uint16_t)i);
    for (int fmt = 0; fmt < 2; ++fmt) {
        const int bit_widths[3] = {3, 4, 8};
        for (int b = 0; b < 3; ++b) {
            const int bits = bit_widths[b];
            const float L = (float)((1 << bits) - 1), qmax = (float)((1 << (bits - 1)) - 1);
            unsigned long long pairs = 0, ties = 0, bad = 0;
            const int count = fmt == 0 ? 0x7c00 : 0x7f80;
            for (int si = 1; si < count; si += stride) {
                const float s = fmt == 0 ? W[si] : bfloat_to_float((uint16_t)si);
                /* scales of binary16 weights: between 2 * 2^-24 / 255 and 2 * 65504 / 7 */
                if (s < 4.6e-10f || s > 18716.0f) continue;
                volatile float rs_v = 1.0f / s;
                const float rs = rs_v;
                const float top = s * L * 0.5f;
                for (int wi = 0; wi < 0x7c00 && W[wi] <= top; ++wi) {
                    const float w = W[wi];
                    volatile float quotient = w / s;
                    float ref = rintf(quotient);
                    volatile float x0_v = w * rs;
                    const float x0 = x0_v;
                    const float x = fmaf(fmaf(-x0, s, w), rs, x0);
                    float got = rintf(x);
                    ref = ref > qmax ? qmax : ref;
                    got = got > qmax ? qmax : got;
                    ++pairs;
                    if (quotient - floorf(quotient) == 0.5f) ++ties;
                    if (got != ref) {
                        if (bad < 5) printf("  mismatch: format %d bits %d s %a w %a: %g vs %g\n", fmt, bits, s, w, ref, got);
                        ++bad;
                    }
                }
            }
            printf("%s scales, %d-bit codes: %llu pairs, %llu exact ties, %llu mismatches\n",
                   fmt == 0 ? "binary16" : "bfloat16", bits, pairs, ties, bad);
            if (bad) ++failed;
        }
    }
    return failed;
}
