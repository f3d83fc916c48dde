/* Host check of an arithmetic identity the quantize kernels rely on (Sec. 3.2: scale = (max - min) / 15).
 *
 * For c = fl(1/15), q0 = fl(r * c), e = fma(-15, q0, r), q = fma(e, c, q0): q == fl(r / 15) for every
 * binary32 r in [lo, hi].  Prints the number of values checked and of mismatches; exit status 1 on any mismatch.
 * usage: div15_check LO_EXP HI_EXP   (checks [2^LO_EXP, 2^HI_EXP]) */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    const float a = ldexpf(1.0f, atoi(argv[1])), b = ldexpf(1.0f, atoi(argv[2]));
    const volatile float fifteen = 15.0f;
    const float c = 1.0f / fifteen;
    uint32_t lo, hi;
    memcpy(&lo, &a, 4);
    memcpy(&hi, &b, 4);
    long bad = 0, plain_bad = 0;
    for (uint32_t u = lo; u <= hi; ++u) {
        float r;
        memcpy(&r, &u, 4);
        const float want = r / fifteen;
        const float q0 = r * c;
        const float e = fmaf(-15.0f, q0, r);
        const float q = fmaf(e, c, q0);
        if (q != want) {
            if (bad < 5) printf("mismatch r=%a got=%a want=%a\n", r, q, want);
            ++bad;
        }
        if (q0 != want) ++plain_bad;
    }
    printf("checked %lu mismatches %ld plain_multiply_mismatches %ld\n", (unsigned long)(hi - lo) + 1, bad, plain_bad);
    return bad != 0;
}
