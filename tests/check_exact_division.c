/* Host check of the identity the GPU quantizers rely on: for one divisor s and
 * its correctly rounded reciprocal r = fl(1/s),
 *     q0 = fl(v * r),  rem = fma(-q0, s, v),  q = fma(rem, r, q0)
 * equals the IEEE single-precision quotient fl(v / s) (Markstein's correction
 * step).  Every pair of finite fp16 values v >= 0, s > 0 is tried (the sign of
 * v carries through every step unchanged), which is every pair the per-token
 * quantizer of Section 2.1 can meet: inputs and scales are both fp16 values.
 * Prints the number of pairs and of mismatches; exit status 1 on any mismatch. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>

static float half_value(int bits)
{
    const int e = (bits >> 10) & 31, m = bits & 1023;
    return e == 0 ? ldexpf((float)m, -24) : ldexpf((float)(m + 1024), e - 25);
}

int main(void)
{
    long pairs = 0, wrong = 0;
#pragma omp parallel for reduction(+ : pairs, wrong) schedule(dynamic, 64)
    for (int sb = 1; sb <= 0x7bff; ++sb) {
        const float s = half_value(sb);
        const float r = 1.0f / s;
        for (int vb = 0; vb <= 0x7bff; ++vb) {
            const float v = half_value(vb);
            const float q0 = v * r;
            const float rem = fmaf(-q0, s, v);
            const float q = fmaf(rem, r, q0);
            ++pairs;
            if (q != v / s) ++wrong;
        }
    }
    printf("%ld %ld\n", pairs, wrong);
    return wrong != 0;
}
