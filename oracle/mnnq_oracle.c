/*
 * CPU oracle for the W4A8 / W4A16 quantized linear layer.
 *
 * TEST INFRASTRUCTURE.  Plain scalar C, one loop nest per definition, no
 * blocking, no intrinsics, no BLAS.  It shares nothing with the HIP library and
 * is only used by tests, the smoke check and the CPU-baseline leg of the
 * benchmark.  OpenMP, when enabled, only distributes whole output rows.
 *
 * What it follows
 *   - Weight codes: the asymmetric quantizer of Section 4.2, Eq. 1 (step =
 *     (w_max - w_min) / (clip_max - clip_min), clip range 0..15 for int4), in
 *     the integer-zero-point form the benchmark configurations name:
 *     group of 64 along K, scale = (max - min)/15, zero = round(-min/scale);
 *     and, second, exactly as Eq. 1 is printed, with the group minimum kept as
 *     a float offset (O6..O8 below; O9, O10 the same with 8-bit codes; O11 these
 *     weights against fp16 activations).
 *   - Activation codes: Section 4.2 says activations are quantized to int8 at
 *     run time; the configurations fix per-token symmetric, scale = max|x|/127.
 *   - Linear: Section 5.1 notation, activations [e, l] x weights [h, l] ->
 *     [e, h]; here e = M, l = K, h = N.
 *
 * All quantizer arithmetic is IEEE binary32, round-to-nearest-even, compiled
 * with -ffp-contract=off.  The floating part of the linear layers is binary64
 * and rounded to binary32 once.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define ORC_GROUP 64

/* O1: weight quantizer (Section 4.2, Eq. 1, integer zero point).
 * W [N,K] row-major fp32 -> q [N,K] one code (0..15) per byte, s [N,G], z [N,G]. */
void orc_quant_weights(const float *W, int64_t N, int64_t K,
                       uint8_t *q, float *s, uint8_t *z)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < G; ++g) {
            const float *w = W + n * K + g * ORC_GROUP;
            uint8_t *qo = q + n * K + g * ORC_GROUP;
            float mn = w[0], mx = w[0];
            for (int k = 1; k < ORC_GROUP; ++k) {
                if (w[k] < mn) mn = w[k];
                if (w[k] > mx) mx = w[k];
            }
            /* A group that does not straddle zero: widen the range to contain
             * zero, so that the zero point stays inside the code range. */
            if (mn > 0.0f) mn = 0.0f;
            if (mx < 0.0f) mx = 0.0f;
            if (mx == mn) { /* only the all-zero group is left here */
                s[n * G + g] = 1.0f;
                z[n * G + g] = 0;
                for (int k = 0; k < ORC_GROUP; ++k) qo[k] = 0;
                continue;
            }
            const float scale = (mx - mn) / 15.0f;
            const float zero = rintf((-mn) / scale);
            s[n * G + g] = scale;
            z[n * G + g] = (uint8_t)zero;
            for (int k = 0; k < ORC_GROUP; ++k) {
                float c = rintf(w[k] / scale) + zero;
                if (c < 0.0f) c = 0.0f;
                if (c > 15.0f) c = 15.0f;
                qo[k] = (uint8_t)c;
            }
        }
    }
}

/* O2: dequantized weight, w^ = (q - z) * s, one binary32 multiply. */
void orc_dequant(const uint8_t *q, const float *s, const uint8_t *z,
                 int64_t N, int64_t K, float *What)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / ORC_GROUP;
            What[n * K + k] = (float)((int)q[n * K + k] - (int)z[n * G + g]) * s[n * G + g];
        }
}

/* O3: per-token symmetric int8 activation quantizer (Section 4.2).
 * x [M,K] fp32 -> xq [M,K] int8, sx [M], xsum [M,G] (may be NULL). */
void orc_quant_act(const float *x, int64_t M, int64_t K,
                   int8_t *xq, float *sx, int32_t *xsum)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const float *xr = x + m * K;
        float amax = 0.0f;
        for (int64_t k = 0; k < K; ++k) {
            const float a = fabsf(xr[k]);
            if (a > amax) amax = a;
        }
        if (amax == 0.0f) {
            sx[m] = 0.0f;
            for (int64_t k = 0; k < K; ++k) xq[m * K + k] = 0;
            if (xsum) for (int64_t g = 0; g < G; ++g) xsum[m * G + g] = 0;
            continue;
        }
        const float scale = amax / 127.0f;
        sx[m] = scale;
        for (int64_t g = 0; g < G; ++g) {
            int32_t acc = 0;
            for (int k = 0; k < ORC_GROUP; ++k) {
                float c = rintf(xr[g * ORC_GROUP + k] / scale);
                if (c < -127.0f) c = -127.0f;
                if (c > 127.0f) c = 127.0f;
                const int8_t v = (int8_t)c;
                xq[m * K + g * ORC_GROUP + k] = v;
                acc += v;
            }
            if (xsum) xsum[m * G + g] = acc;
        }
    }
}

/* O4: W4A8 linear.  I[m,n,g] = sum_{k in g} xq[m,k] * (q[n,k] - z[n,g]) exactly
 * in int32; y[m,n] = sx[m] * sum_g s[n,g] * I[m,n,g] (+ bias[n]) in binary64,
 * rounded once.  acc ([M,N,G]) and bias may be NULL. */
void orc_linear_w4a8(const int8_t *xq, const float *sx,
                     const uint8_t *q, const float *s, const uint8_t *z,
                     const float *bias, int64_t M, int64_t N, int64_t K,
                     int32_t *acc, float *y)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                const int8_t *a = xq + m * K + g * ORC_GROUP;
                const uint8_t *b = q + n * K + g * ORC_GROUP;
                const int32_t zero = z[n * G + g];
                int32_t I = 0;
                for (int k = 0; k < ORC_GROUP; ++k)
                    I += (int32_t)a[k] * ((int32_t)b[k] - zero);
                if (acc) acc[(m * N + n) * G + g] = I;
                sum += (double)s[n * G + g] * (double)I;
            }
            double r = (double)sx[m] * sum;
            if (bias) r += (double)bias[n];
            if (y) y[m * N + n] = (float)r;
        }
    }
}

/* IEEE binary16 bits -> binary32 value (exact widening). */
static float orc_half_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const int32_t e = (h >> 10) & 0x1f;
    const uint32_t m = h & 0x3ffu;
    float mag;
    if (e == 0)        mag = ldexpf((float)m, -24);              /* zero, subnormal */
    else if (e == 31)  mag = m ? NAN : INFINITY;
    else               mag = ldexpf((float)(m | 0x400u), e - 25);
    uint32_t bits;
    memcpy(&bits, &mag, 4);
    bits |= sign;
    memcpy(&mag, &bits, 4);
    return mag;
}

/* O5: W4A16 linear (Section 4.2: int4 weights, fp16 activations on the GPU
 * path).  y[m,n] = sum_k float(x16[m,k]) * w^[n,k] (+ bias[n]), w^ from O2 in
 * binary32, products and sum in binary64, rounded once. */
void orc_linear_w4a16(const uint16_t *x16,
                      const uint8_t *q, const float *s, const uint8_t *z,
                      const float *bias, int64_t M, int64_t N, int64_t K, float *y)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t g = k / ORC_GROUP;
                const float what = (float)((int)q[n * K + k] - (int)z[n * G + g]) * s[n * G + g];
                sum += (double)orc_half_to_float(x16[m * K + k]) * (double)what;
            }
            if (bias) sum += (double)bias[n];
            y[m * N + n] = (float)sum;
        }
    }
}

/* Sampled rows of O4, so that full-size outputs can be checked one by one:
 * computes acc/y only for the `count` (m,n) pairs listed in ms[], ns[]. */
void orc_linear_w4a8_sampled(const int8_t *xq, const float *sx,
                             const uint8_t *q, const float *s, const uint8_t *z,
                             const float *bias, int64_t M, int64_t N, int64_t K,
                             const int64_t *ms, const int64_t *ns, int64_t count,
                             int32_t *acc /* [count,G] or NULL */, float *y /* [count] */)
{
    const int64_t G = K / ORC_GROUP;
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t m = ms[i], n = ns[i];
        double sum = 0.0;
        for (int64_t g = 0; g < G; ++g) {
            int32_t I = 0;
            const int32_t zero = z[n * G + g];
            for (int k = 0; k < ORC_GROUP; ++k)
                I += (int32_t)xq[m * K + g * ORC_GROUP + k] *
                     ((int32_t)q[n * K + g * ORC_GROUP + k] - zero);
            if (acc) acc[i * G + g] = I;
            sum += (double)s[n * G + g] * (double)I;
        }
        double r = (double)sx[m] * sum;
        if (bias) r += (double)bias[n];
        y[i] = (float)r;
    }
}

/* Sampled rows of O5, same purpose. */
void orc_linear_w4a16_sampled(const uint16_t *x16,
                              const uint8_t *q, const float *s, const uint8_t *z,
                              const float *bias, int64_t M, int64_t N, int64_t K,
                              const int64_t *ms, const int64_t *ns, int64_t count, float *y)
{
    const int64_t G = K / ORC_GROUP;
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t m = ms[i], n = ns[i];
        double sum = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / ORC_GROUP;
            const float what = (float)((int)q[n * K + k] - (int)z[n * G + g]) * s[n * G + g];
            sum += (double)orc_half_to_float(x16[m * K + k]) * (double)what;
        }
        if (bias) sum += (double)bias[n];
        y[i] = (float)sum;
    }
}

/* ---- Eq. 1 taken literally: the group minimum stays a float offset --------
 *
 * Section 4.2, Eq. 1 with clip_min = 0, clip_max = 15:
 *     q = round((w - w_min) / step),  step = (w_max - w_min) / 15,
 * and the weight it stands for is w^ = q * step + w_min.  There is no integer
 * zero point: the stored parameters of a group are (step, w_min). */

/* O6: weight quantizer, float-minimum form.
 * W [N,K] -> q [N,K] (0..15), s [N,G] (step), wmin [N,G].  A constant group has
 * step 1 and all codes 0, so that w^ = w_min is exact. */
void orc_quant_weights_minf(const float *W, int64_t N, int64_t K,
                            uint8_t *q, float *s, float *wmin)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < G; ++g) {
            const float *w = W + n * K + g * ORC_GROUP;
            uint8_t *qo = q + n * K + g * ORC_GROUP;
            float mn = w[0], mx = w[0];
            for (int k = 1; k < ORC_GROUP; ++k) {
                if (w[k] < mn) mn = w[k];
                if (w[k] > mx) mx = w[k];
            }
            wmin[n * G + g] = mn;
            if (mx == mn) {
                s[n * G + g] = 1.0f;
                for (int k = 0; k < ORC_GROUP; ++k) qo[k] = 0;
                continue;
            }
            const float step = (mx - mn) / 15.0f;
            s[n * G + g] = step;
            for (int k = 0; k < ORC_GROUP; ++k) {
                float c = rintf((w[k] - mn) / step);
                if (c < 0.0f) c = 0.0f;
                if (c > 15.0f) c = 15.0f;
                qo[k] = (uint8_t)c;
            }
        }
    }
}

/* O7: the weight a code stands for, w^ = q * step + w_min, evaluated in binary64
 * (the product is exact there) and rounded to binary32 once. */
void orc_dequant_minf(const uint8_t *q, const float *s, const float *wmin,
                      int64_t N, int64_t K, float *What)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n)
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / ORC_GROUP;
            What[n * K + k] = (float)((double)q[n * K + k] * (double)s[n * G + g] + (double)wmin[n * G + g]);
        }
}

/* O8: W4A8 linear on float-minimum weights.
 *   A[m,n,g]  = sum_{k in g} xq[m,k] * q[n,k]           (int32, exact)
 *   xs[m,g]   = sum_{k in g} xq[m,k]                    (int32, exact)
 *   y[m,n]    = sx[m] * sum_g (s[n,g] * A[m,n,g] + wmin[n,g] * xs[m,g]) (+ bias[n])
 * which is sum_k (sx xq)[m,k] * w^[n,k] with w^ = q s + wmin.  binary64, rounded once. */
void orc_linear_w4a8_minf(const int8_t *xq, const float *sx,
                          const uint8_t *q, const float *s, const float *wmin,
                          const float *bias, int64_t M, int64_t N, int64_t K,
                          int32_t *acc, float *y)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t g = 0; g < G; ++g) {
                const int8_t *a = xq + m * K + g * ORC_GROUP;
                const uint8_t *b = q + n * K + g * ORC_GROUP;
                int32_t A = 0, xs = 0;
                for (int k = 0; k < ORC_GROUP; ++k) {
                    A += (int32_t)a[k] * (int32_t)b[k];
                    xs += (int32_t)a[k];
                }
                if (acc) acc[(m * N + n) * G + g] = A;
                sum += (double)s[n * G + g] * (double)A + (double)wmin[n * G + g] * (double)xs;
            }
            double r = (double)sx[m] * sum;
            if (bias) r += (double)bias[n];
            if (y) y[m * N + n] = (float)r;
        }
    }
}

/* Sampled (m,n) pairs of O8. */
void orc_linear_w4a8_minf_sampled(const int8_t *xq, const float *sx,
                                  const uint8_t *q, const float *s, const float *wmin,
                                  const float *bias, int64_t M, int64_t N, int64_t K,
                                  const int64_t *ms, const int64_t *ns, int64_t count,
                                  int32_t *acc /* [count,G] or NULL */, float *y /* [count] */)
{
    const int64_t G = K / ORC_GROUP;
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t m = ms[i], n = ns[i];
        double sum = 0.0;
        for (int64_t g = 0; g < G; ++g) {
            int32_t A = 0, xs = 0;
            for (int k = 0; k < ORC_GROUP; ++k) {
                const int32_t a = xq[m * K + g * ORC_GROUP + k];
                A += a * (int32_t)q[n * K + g * ORC_GROUP + k];
                xs += a;
            }
            if (acc) acc[i * G + g] = A;
            sum += (double)s[n * G + g] * (double)A + (double)wmin[n * G + g] * (double)xs;
        }
        double r = (double)sx[m] * sum;
        if (bias) r += (double)bias[n];
        y[i] = (float)r;
    }
}

/* ---- int8 weights (Section 4.2: parameters are quantized to int4 or int8; the
 * LM head is prioritised for int8), Eq. 1 as printed with clip range 0..255:
 *     q = round((w - w_min) / step),  step = (w_max - w_min) / 255,  w^ = q * step + w_min. */

/* O9: 8-bit weight quantizer.  W [N,K] -> q [N,K] (0..255), s [N,G] (step), wmin [N,G]. */
void orc_quant_weights8(const float *W, int64_t N, int64_t K,
                        uint8_t *q, float *s, float *wmin)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t g = 0; g < G; ++g) {
            const float *w = W + n * K + g * ORC_GROUP;
            uint8_t *qo = q + n * K + g * ORC_GROUP;
            float mn = w[0], mx = w[0];
            for (int k = 1; k < ORC_GROUP; ++k) {
                if (w[k] < mn) mn = w[k];
                if (w[k] > mx) mx = w[k];
            }
            wmin[n * G + g] = mn;
            if (mx == mn) {
                s[n * G + g] = 1.0f;
                for (int k = 0; k < ORC_GROUP; ++k) qo[k] = 0;
                continue;
            }
            const float step = (mx - mn) / 255.0f;
            s[n * G + g] = step;
            for (int k = 0; k < ORC_GROUP; ++k) {
                float c = rintf((w[k] - mn) / step);
                if (c < 0.0f) c = 0.0f;
                if (c > 255.0f) c = 255.0f;
                qo[k] = (uint8_t)c;
            }
        }
    }
}

/* O10: W8A8 linear.  The code range only enters through q, so this is O8 on 8-bit codes:
 *   A[m,n,g] = sum_{k in g} xq[m,k] * q[n,k],  xs[m,g] = sum_{k in g} xq[m,k]   (int32, exact:
 *   |A| <= 64 * 127 * 255 < 2^21)
 *   y[m,n] = sx[m] * sum_g (s[n,g] * A[m,n,g] + wmin[n,g] * xs[m,g]) (+ bias[n]). */
void orc_linear_w8a8(const int8_t *xq, const float *sx,
                     const uint8_t *q, const float *s, const float *wmin,
                     const float *bias, int64_t M, int64_t N, int64_t K,
                     int32_t *acc, float *y)
{
    orc_linear_w4a8_minf(xq, sx, q, s, wmin, bias, M, N, K, acc, y);
}

void orc_linear_w8a8_sampled(const int8_t *xq, const float *sx,
                             const uint8_t *q, const float *s, const float *wmin,
                             const float *bias, int64_t M, int64_t N, int64_t K,
                             const int64_t *ms, const int64_t *ns, int64_t count,
                             int32_t *acc, float *y)
{
    orc_linear_w4a8_minf_sampled(xq, sx, q, s, wmin, bias, M, N, K, ms, ns, count, acc, y);
}

/* O11: fp16 activations on float-minimum weights (Section 4.2: the GPU path combines the
 * quantized weights with fp16 activations; Eq. 1 gives the weight a code stands for).
 *   y[m,n] = sum_k float(x16[m,k]) * (q[n,k] * s[n,g] + wmin[n,g]) (+ bias[n])
 * for 4-bit (0..15) and 8-bit (0..255) codes alike; every product and the sum in binary64,
 * rounded once. */
void orc_linear_a16_minf(const uint16_t *x16,
                         const uint8_t *q, const float *s, const float *wmin,
                         const float *bias, int64_t M, int64_t N, int64_t K, float *y)
{
    const int64_t G = K / ORC_GROUP;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        for (int64_t m = 0; m < M; ++m) {
            double sum = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                const int64_t g = k / ORC_GROUP;
                const double what = (double)q[n * K + k] * (double)s[n * G + g] + (double)wmin[n * G + g];
                sum += (double)orc_half_to_float(x16[m * K + k]) * what;
            }
            if (bias) sum += (double)bias[n];
            y[m * N + n] = (float)sum;
        }
    }
}

/* Sampled (m,n) pairs of O11. */
void orc_linear_a16_minf_sampled(const uint16_t *x16,
                                 const uint8_t *q, const float *s, const float *wmin,
                                 const float *bias, int64_t M, int64_t N, int64_t K,
                                 const int64_t *ms, const int64_t *ns, int64_t count, float *y)
{
    const int64_t G = K / ORC_GROUP;
    (void)M; (void)N;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < count; ++i) {
        const int64_t m = ms[i], n = ns[i];
        double sum = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            const int64_t g = k / ORC_GROUP;
            const double what = (double)q[n * K + k] * (double)s[n * G + g] + (double)wmin[n * G + g];
            sum += (double)orc_half_to_float(x16[m * K + k]) * what;
        }
        if (bias) sum += (double)bias[n];
        y[i] = (float)sum;
    }
}

int orc_omp_enabled(void)
{
#ifdef _OPENMP
    return 1;
#else
    return 0;
#endif
}
