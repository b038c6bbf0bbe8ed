/*
 * FlexQ oracle -- TEST INFRASTRUCTURE, not the product.
 *
 * A plain, slow CPU statement of what the W6A6 / W6A8 quantized linear layer
 * computes.  Only the tests, the smoke check and the benchmark's cpu_baseline
 * leg may call it; the GPU library never does, and the two share no code.
 *
 * What the paper fixes and where:
 *   - symmetric quantization without zero point, for weights and activations
 *     (Section 2.1, "Quantization of Large Language Models");
 *   - one scale per group of consecutive elements along a channel, group 128
 *     by default (Section 4.1.1, "Weight & Activation Fine-grained Group
 *     Quantization"); a whole row as one group gives the per-channel /
 *     per-token case;
 *   - the integer product of the quantized operands as a sum of bit-plane
 *     products weighted by 2^(s+t) (Section 4.2, Eq. 4 and Eq. 5);
 *   - dequantization fused into the product: each group's integer partial
 *     product is multiplied by that group's weight scale and activation
 *     scale and the results are summed (Section 4.2, Eq. 7; Section 4.3.4),
 *     scales being stored as fp16.
 *
 * Readings taken where the paper is silent (listed in the design notes too):
 *   scale = absmax / (2^(b-1) - 1), rounded to fp16 BEFORE it is used, with
 *   1.0 substituted when absmax (or the rounded scale) is zero; the quotient
 *   v / scale is an IEEE fp32 division rounded half-to-even to an integer and
 *   clamped to [-2^(b-1), 2^(b-1) - 1]; negative values are two's complement,
 *   so the top bit plane carries weight -2^(b-1); Eq. 7 as printed drops the
 *   2^(s+t) factor that Eq. 5 has -- it is restored here; dequantization is
 *   done in fp64 with a single final rounding to fp16.
 *
 * Every function is pinned by tests that do not go through this file's own
 * arithmetic: numpy's integer matmul and fp16 conversion, brute force on tiny
 * inputs, the paper's worked 2-bit x 4-bit expansion (Eq. 3), closed forms
 * and crafted ties.  The paper prints no numeric quantization example, so the
 * scale formula, rounding mode and clamp are fixed by the benchmark spec and
 * the invariants only.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see build.py).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------ fp16 */

/* fp16 bit pattern -> exact double. */
double flexq_oracle_f16_to_f64(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);               /* zero and subnormals      */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(1024 + m), e - 25);   /* 1.m * 2^(e-15)           */
    return sign ? -v : v;
}

/* double -> nearest fp16 bit pattern, ties to even, in ONE rounding
 * (never through float: a double rounding could move a tie). */
uint16_t flexq_oracle_f64_to_f16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0u;
    if (isnan(x))
        return (uint16_t)(sign | 0x7e00u);
    double a = fabs(x);
    if (a >= 65520.0)                            /* halfway to 2^16 and up   */
        return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0)
        return sign;
    int e;
    (void)frexp(a, &e);                          /* a = f * 2^e, f in [.5,1) */
    e -= 1;                                      /* a in [2^e, 2^(e+1))      */
    if (e < -14)
        e = -14;                                 /* subnormal spacing        */
    /* spacing of fp16 numbers in this binade is 2^(e-10) */
    double n = ldexp(a, 10 - e);                 /* exact: power-of-two scale */
    double r = nearbyint(n);                     /* default mode: half-even  */
    /* r in [0, 2048]; r == 2048 means the value rounded up to 2^(e+1) */
    if (r >= 2048.0) {
        r = 1024.0;
        e += 1;
    }
    if (r < 1024.0)                              /* only possible at e = -14 */
        return (uint16_t)(sign | (uint16_t)r);   /* subnormal or zero        */
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)(r - 1024.0));
}

/* ------------------------------------------------------------- quantizer */

/*
 * Symmetric quantization of `rows` rows of length L, one scale per group of G
 * consecutive elements (G divides L; G == L is the per-channel / per-token
 * case).  bits is 6 or 8.  q gets rows*L codes, s gets rows*(L/G) fp16 scales.
 * (Section 2.1; Section 4.1.1.)
 */
void flexq_oracle_quantize(const float *v, int64_t rows, int64_t L, int64_t G,
                           int bits, int8_t *q, uint16_t *s)
{
    const int qmax = (1 << (bits - 1)) - 1;
    const int qmin = -(1 << (bits - 1));
    const int64_t ng = L / G;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t g = 0; g < ng; ++g) {
            const float *vg = v + r * L + g * G;
            float amax = 0.0f;
            for (int64_t i = 0; i < G; ++i) {
                float a = fabsf(vg[i]);
                if (a > amax)
                    amax = a;
            }
            float s32 = amax / (float)qmax;
            uint16_t sh = flexq_oracle_f64_to_f16((double)s32);
            float sf = (float)flexq_oracle_f16_to_f64(sh);
            if (amax == 0.0f || sf == 0.0f) {
                sh = 0x3c00u;                    /* 1.0 */
                sf = 1.0f;
            }
            s[r * ng + g] = sh;
            for (int64_t i = 0; i < G; ++i) {
                float quo = vg[i] / sf;          /* one fp32 division        */
                float rn = nearbyintf(quo);      /* half-to-even             */
                int qi;
                if (rn > (float)qmax)
                    qi = qmax;
                else if (rn < (float)qmin)
                    qi = qmin;
                else
                    qi = (int)rn;
                q[r * L + g * G + i] = (int8_t)qi;
            }
        }
    }
}

/* --------------------------------------------------------- integer product */

/*
 * acc[m][n][g] = sum over the g-th group of G consecutive k of
 * xq[m][k] * wq[n][k], accumulated in int64 (G == K gives the whole product).
 * Returns the number of (m, n) whose total over all groups does not fit int32.
 * (Section 4.2: the product the bit-plane sum of Eq. 5 reconstructs.)
 */
int64_t flexq_oracle_matmul(const int8_t *xq, const int8_t *wq, int64_t M,
                            int64_t N, int64_t K, int64_t G, int64_t *acc)
{
    const int64_t ng = K / G;
    int64_t overflow = 0;
#pragma omp parallel for schedule(static) reduction(+ : overflow)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            int64_t total = 0;
            for (int64_t g = 0; g < ng; ++g) {
                int64_t sum = 0;
                for (int64_t k = g * G; k < (g + 1) * G; ++k)
                    sum += (int64_t)xq[m * K + k] * (int64_t)wq[n * K + k];
                acc[(m * N + n) * ng + g] = sum;
                total += sum;
            }
            if (total > INT32_MAX || total < INT32_MIN)
                overflow += 1;
        }
    }
    return overflow;
}

/*
 * The same product written the paper's way (Section 4.2, Eq. 4 and Eq. 5):
 * split W into p one-bit planes and X into q one-bit planes, multiply every
 * pair of planes as 0/1 matrices, and add the p*q results weighted by
 * 2^(s+t).  With is_signed != 0 the inputs are two's complement and the top
 * plane of each operand carries weight -2^(bits-1) (the paper's Eq. 1-2 only
 * write the unsigned case); with is_signed == 0 the inputs must be
 * non-negative and below 2^p / 2^q.  acc is [M][N], whole-K.
 */
void flexq_oracle_bitplane_matmul(const int8_t *xq, const int8_t *wq,
                                  int64_t M, int64_t N, int64_t K, int p,
                                  int q, int is_signed, int64_t *acc)
{
    for (int64_t i = 0; i < M * N; ++i)
        acc[i] = 0;
    for (int s = 0; s < p; ++s) {
        for (int t = 0; t < q; ++t) {
            int64_t weight = (int64_t)1 << (s + t);
            if (is_signed && (s == p - 1) != (t == q - 1))
                weight = -weight;                /* exactly one top plane    */
            for (int64_t m = 0; m < M; ++m) {
                for (int64_t n = 0; n < N; ++n) {
                    int64_t ones = 0;            /* one 1-bit product Y^(s,t) */
                    for (int64_t k = 0; k < K; ++k) {
                        int wb = ((uint8_t)wq[n * K + k] >> s) & 1;
                        int xb = ((uint8_t)xq[m * K + k] >> t) & 1;
                        ones += wb & xb;
                    }
                    acc[m * N + n] += weight * ones;
                }
            }
        }
    }
}

/* ------------------------------------------------------------ dequantize */

/*
 * y[m][n] = fp16( sx[m] * sum_g sw[n][g] * acc[m][n][g] ), all in fp64 with
 * one final rounding.  ng == 1 is the per-channel case, where the fp64
 * product is exact (31 + 11 + 11 bits).  (Section 4.2, Eq. 7 with the
 * per-token activation scale factored out; Section 4.3.4.)
 */
void flexq_oracle_dequant(const int64_t *acc, int64_t M, int64_t N, int64_t ng,
                          const uint16_t *sx, const uint16_t *sw, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t g = 0; g < ng; ++g)
                sum += flexq_oracle_f16_to_f64(sw[n * ng + g]) *
                       (double)acc[(m * N + n) * ng + g];
            double val = flexq_oracle_f16_to_f64(sx[m]) * sum;
            y[m * N + n] = flexq_oracle_f64_to_f16(val);
        }
    }
}

/*
 * Eq. 7 in full: both operands carry a scale per group,
 * y[m][n] = fp16( sum_g sx[m][g] * sw[n][g] * acc[m][n][g] ).
 */
void flexq_oracle_dequant_xgroup(const int64_t *acc, int64_t M, int64_t N,
                                 int64_t ng, const uint16_t *sx,
                                 const uint16_t *sw, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t g = 0; g < ng; ++g)
                sum += flexq_oracle_f16_to_f64(sx[m * ng + g]) *
                       flexq_oracle_f16_to_f64(sw[n * ng + g]) *
                       (double)acc[(m * N + n) * ng + g];
            y[m * N + n] = flexq_oracle_f64_to_f16(sum);
        }
    }
}

/* ------------------------------------------------- 6-bit field round trip */

/*
 * Reference statement of "weights are stored at 6 bits": the densest possible
 * form, codes laid end to end, 4 codes in 3 bytes, little-endian bit order.
 * This is NOT the GPU library's layout (that one is opaque); it pins the size
 * (exactly 0.75 bytes per weight) and that 6 bits hold every code in
 * [-32, 31] losslessly.  (Section 4.3.1, "Bit-level Data Packing".)
 */
void flexq_oracle_pack6_dense(const int8_t *wq, int64_t count, uint8_t *out)
{
    memset(out, 0, (size_t)(count * 6 / 8));
    for (int64_t i = 0; i < count; ++i) {
        uint32_t code = (uint32_t)wq[i] & 63u;
        for (int b = 0; b < 6; ++b) {
            int64_t bit = i * 6 + b;
            if ((code >> b) & 1u)
                out[bit >> 3] |= (uint8_t)(1u << (bit & 7));
        }
    }
}

void flexq_oracle_unpack6_dense(const uint8_t *in, int64_t count, int8_t *wq)
{
    for (int64_t i = 0; i < count; ++i) {
        int code = 0;
        for (int b = 0; b < 6; ++b) {
            int64_t bit = i * 6 + b;
            code |= ((in[bit >> 3] >> (bit & 7)) & 1) << b;
        }
        wq[i] = (int8_t)(code >= 32 ? code - 64 : code);
    }
}

/* --------------------------------------- producers of the activations */

/*
 * The paper fuses the activation quantizer into the kernel that produces the
 * activations: the normalization before the QKV and gate/up projections, and the
 * activation function before the down projection (Section 4.1.3, "FlexQ System
 * Runtime").  These two functions state what those producers output BEFORE the
 * quantizer, as fp16 (what the unfused pipeline would hand to the quantizer):
 *
 *   RMS normalization (LLaMA's):  h[m][k] = fp16( x[m][k] / sqrt(mean_k x^2 + eps) * gamma[k] )
 *   gated SiLU ("SwiGLU"):        h[m][f] = fp16( g / (1 + exp(-g)) * u ),
 *                                  g = gu[m][f], u = gu[m][F + f]   (fused gate|up layout)
 *
 * both evaluated in fp64 with one final rounding.  The paper does not specify
 * either formula beyond naming the layers; they are the public definitions of
 * the LLaMA architecture it evaluates.
 */
void flexq_oracle_rmsnorm(const uint16_t *x, const uint16_t *gamma, int64_t M,
                          int64_t K, double eps, uint16_t *h)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double v = flexq_oracle_f16_to_f64(x[m * K + k]);
            ss += v * v;
        }
        double inv = 1.0 / sqrt(ss / (double)K + eps);
        for (int64_t k = 0; k < K; ++k)
            h[m * K + k] = flexq_oracle_f64_to_f16(flexq_oracle_f16_to_f64(x[m * K + k]) * inv *
                                                   flexq_oracle_f16_to_f64(gamma[k]));
    }
}

void flexq_oracle_swiglu(const uint16_t *gu, int64_t M, int64_t F, uint16_t *h)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t f = 0; f < F; ++f) {
            double g = flexq_oracle_f16_to_f64(gu[m * 2 * F + f]);
            double u = flexq_oracle_f16_to_f64(gu[m * 2 * F + F + f]);
            h[m * F + f] = flexq_oracle_f64_to_f16(g / (1.0 + exp(-g)) * u);
        }
    }
}

int flexq_oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
