/* Host check of the identity the compress kernels use for the group scale (Sec. 3.2, linear quantisation:
 * scale = range / levels):   q0 = a * y,  q = fma(fma(-L, q0, a), y, q0),  y = the binary32 nearest 1 / L,
 * equals the correctly rounded binary32 quotient a / L for L = 3, 15, 255.
 * Usage: scale_division_check STRIDE  - every STRIDE-th binary32 bit pattern in (0, 2^17] (1 = all of them,
 * about a minute on eight cores), plus every difference of two binary16 values whose exponents differ by
 * at most one.  Prints the number of mismatches per divisor; exit status 1 if there is any. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static float from_bits(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

static float half_value(uint32_t h) {            /* positive binary16 bit pattern -> value */
    const int e = (int)(h >> 10) & 31, m = (int)(h & 1023);
    return e ? ldexpf((float)(1024 + m), e - 25) : ldexpf((float)m, -24);
}

static int differs(float a, float L, float y) {
    const float q0 = a * y;
    const float q = fmaf(fmaf(-L, q0, a), y, q0);
    const float ref = a / L;
    return memcmp(&q, &ref, 4) != 0;
}

int main(int argc, char** argv) {
    const uint32_t stride = argc > 1 ? (uint32_t)strtoul(argv[1], NULL, 10) : 1;
    const float Ls[3] = {3.0f, 15.0f, 255.0f};
    uint32_t top;
    const float two17 = 131072.0f;
    long total = 0;
    memcpy(&top, &two17, 4);
    if (!stride) return 2;
    for (int li = 0; li < 3; ++li) {
        const float L = Ls[li];
        volatile float yv = 1.0f / L;
        const float y = yv;
        long bad = 0;
#pragma omp parallel for reduction(+ : bad) schedule(static)
        for (uint32_t u = 1; u <= top / stride; ++u) bad += differs(from_bits(u * stride), L, y);
        bad += differs(two17, L, y);
#pragma omp parallel for reduction(+ : bad) schedule(static)
        for (uint32_t hi = 1; hi < 0x7c00; ++hi) {
            const float a = half_value(hi);
            const uint32_t first = hi > 2048 ? hi - 2048 : 0;     /* the two binades below hi's */
            for (uint32_t lo = first; lo < hi; ++lo) {
                bad += differs(a - half_value(lo), L, y);         /* minimum and maximum of one sign */
                bad += differs(a + half_value(lo), L, y);         /* minimum negative */
            }
        }
        printf("levels %g: %ld mismatches\n", L, bad);
        total += bad;
    }
    return total ? 1 : 0;
}
