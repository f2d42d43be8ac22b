/*
 * CPU oracle for the per-layer local-metric sensitivity pass of QuantuneV2
 * (arXiv 2501.07161).  TEST INFRASTRUCTURE ONLY: it is called by the tests, by
 * the smoke check and by the benchmark's cpu_baseline leg, never by the
 * product path.  It shares no code, header, table or helper with the HIP
 * library; it is written directly from the paper's definitions.
 *
 * Plain sequential loops, one tensor (or one channel) at a time.  Every
 * accumulation is fp64.  The only fp32 roundings are the ones the quantizer
 * itself is defined with (fp32 scale, fp32 multiply, round-half-to-even,
 * clamp to [-128,127]); they are spelled out where they happen.
 *
 * Build: gcc -O2 -std=c11 -fPIC -shared -ffp-contract=off -fno-fast-math
 * (no contraction, no value-changing optimisation; default rounding mode).
 *
 * Readings of the paper taken here (the paper is silent or inconsistent):
 *  - Sec. 2.1 Eq. 1-3 describe an unsigned code offset by a real x_min; the
 *    task fixes signed int8 codes with an integer zero-point, which is the
 *    same uniform grid shifted by at most half a step.
 *  - The calibrated range is widened to contain 0 so that an integer
 *    zero-point inside [-128,127] always exists and exact zeros (post-ReLU
 *    activations) stay exact.
 *  - Sec. 4 Eq. 4 defines S = (2^(b-1)-1)/max|W| (codes per unit) while Eq. 5
 *    divides by S; Eq. 4's S is read as the multiplier.  The reported `scale`
 *    is the step (max|W|/127, or (hi-lo)/255 for Eq. 2 with N = 256) and the
 *    per-element operation is one fp32 multiply by inv_scale = 1.0f/scale.
 *  - `round` is round-half-to-even; the zero-point is added after rounding,
 *    in integers.
 *  - Sec. 6.1 Eq. 7 is printed garbled; MSE is the mean squared difference
 *    between the original and the dequantized values, as its prose says.
 *  - Eq. 6: P_signal / P_noise is sum(x^2) / sum((x - xhat)^2).
 */
#include <math.h>
#include <stdint.h>
#include <float.h>

/* Sec. 2.1 Eq. 1-2: x_min and x_max of a tensor.  NaNs never win a comparison
 * and are therefore ignored; an empty or all-NaN tensor gives (+inf, -inf).
 * A result of -0.0 is reported as +0.0. */
void orc_minmax(const float *x, int64_t n, float *mn_out, float *mx_out)
{
    float mn = INFINITY, mx = -INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        if (x[i] < mn) mn = x[i];
        if (x[i] > mx) mx = x[i];
    }
    *mn_out = mn + 0.0f;
    *mx_out = mx + 0.0f;
}

/* Brute-force argmin/argmax (first occurrence), used by the pins. */
void orc_argminmax(const float *x, int64_t n, int64_t *imin, int64_t *imax)
{
    int64_t a = -1, b = -1;
    for (int64_t i = 0; i < n; ++i) {
        if (a < 0 || x[i] < x[a]) a = i;
        if (b < 0 || x[i] > x[b]) b = i;
    }
    *imin = a;
    *imax = b;
}

/* Tensor statistics used as local metrics (abstract; Sec. 4 step 1):
 * sum(x) and sum(x^2) in fp64. */
void orc_moments(const float *x, int64_t n, double *sum_x, double *sum_x2)
{
    double s = 0.0, s2 = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)x[i];
        s += v;
        s2 += v * v;
    }
    *sum_x = s;
    *sum_x2 = s2;
}

/* Population variance, two-pass, fp64. */
double orc_variance(const float *x, int64_t n)
{
    if (n <= 0) return 0.0;
    double s = 0.0;
    for (int64_t i = 0; i < n; ++i) s += (double)x[i];
    double mean = s / (double)n;
    double acc = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double d = (double)x[i] - mean;
        acc += d * d;
    }
    return acc / (double)n;
}

static int32_t clamp_i32(int64_t v, int32_t lo, int32_t hi)
{
    if (v < lo) return lo;
    if (v > hi) return hi;
    return (int32_t)v;
}

/* Asymmetric per-tensor parameters: Sec. 2.1 Eq. 2 with N = 256 levels on the
 * range widened to contain zero.  All arithmetic is fp32, one rounding per
 * operation.  Degenerate range (all zeros) or a sub-normal step: scale = 1. */
void orc_params_asym(float mn, float mx, float *scale, float *inv_scale, int32_t *zp)
{
    float lo = mn < 0.0f ? mn : 0.0f;
    float hi = mx > 0.0f ? mx : 0.0f;
    float range = hi - lo;
    float s = range / 255.0f;
    if (!(s >= FLT_MIN)) {
        *scale = 1.0f;
        *inv_scale = 1.0f;
        *zp = 0;
        return;
    }
    float inv = 1.0f / s;
    float prod = lo * inv;
    float z = -128.0f - prod;
    *scale = s;
    *inv_scale = inv;
    *zp = clamp_i32((int64_t)llrintf(z), -128, 127);
}

/* Symmetric parameters: Sec. 4 Eq. 4 with b = 8 (127 codes per max|W|). */
void orc_params_sym(float mn, float mx, float *scale, float *inv_scale, int32_t *zp)
{
    float absmax = fabsf(mn) > fabsf(mx) ? fabsf(mn) : fabsf(mx);
    float s = absmax / 127.0f;
    *zp = 0;
    if (!(s >= FLT_MIN)) {
        *scale = 1.0f;
        *inv_scale = 1.0f;
        return;
    }
    *scale = s;
    *inv_scale = 1.0f / s;
}

/* Sec. 2.1 Eq. 1 / Sec. 4 Eq. 5: code = clamp(rne(x * inv_scale) + zp). */
void orc_quantize(const float *x, int64_t n, float inv_scale, int32_t zp, int8_t *q)
{
    for (int64_t i = 0; i < n; ++i) {
        float t = x[i] * inv_scale;          /* fp32 multiply */
        if (t > 1.0e9f) t = 1.0e9f;          /* keep the integer conversion defined */
        if (t < -1.0e9f) t = -1.0e9f;
        int64_t r = (int64_t)llrintf(t);     /* round half to even */
        q[i] = (int8_t)clamp_i32(r + (int64_t)zp, -128, 127);
    }
}

/* Sec. 2.1 Eq. 3: xhat = (code - zp) * scale, one fp32 multiply. */
void orc_dequantize(const int8_t *q, int64_t n, float scale, int32_t zp, float *xhat)
{
    for (int64_t i = 0; i < n; ++i) {
        float k = (float)((int32_t)q[i] - zp);   /* exact */
        xhat[i] = k * scale;
    }
}

/* Signal and noise energies of Sec. 6.1 Eq. 6-7 between an original tensor and
 * its quantized counterpart: sum(x^2) and sum((x - xhat)^2), fp64. */
void orc_error_sums(const float *x, const float *xhat, int64_t n,
                    double *sum_x2, double *sum_e2)
{
    double s2 = 0.0, e2 = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double v = (double)x[i];
        double e = v - (double)xhat[i];
        s2 += v * v;
        e2 += e * e;
    }
    *sum_x2 = s2;
    *sum_e2 = e2;
}

/* Sec. 6.1 Eq. 7. */
double orc_mse(double sum_e2, int64_t n)
{
    return sum_e2 / (double)n;
}

/* Sec. 6.1 Eq. 6, in dB.  No noise => +inf (also when both energies are 0). */
double orc_sqnr_db(double sum_x2, double sum_e2)
{
    if (sum_e2 == 0.0) return INFINITY;
    return 10.0 * log10(sum_x2 / sum_e2);
}

/* Sec. 6.1 Eq. 8: the three sums behind the cosine similarity of two tensors,
 * sum(a*b), sum(a^2), sum(b^2), fp64. */
void orc_cosine_sums(const float *a, const float *b, int64_t n,
                     double *sab, double *saa, double *sbb)
{
    double xy = 0.0, xx = 0.0, yy = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double x = (double)a[i], y = (double)b[i];
        xy += x * y;
        xx += x * x;
        yy += y * y;
    }
    *sab = xy;
    *saa = xx;
    *sbb = yy;
}

/* Sec. 5, calibration stage: histogram of a tensor's values over [lo, hi] with
 * nbins equal bins.  The paper gives no binning rule; reading taken (fp32, one
 * rounding per step, so that the bin of every element is well defined):
 *   inv_w = nbins / (hi - lo)          (0 when hi - lo is not a positive finite number)
 *   bin   = clamp(floor((x - lo) * inv_w), 0, nbins - 1)
 * Values outside [lo, hi] fall into the edge bins. */
void orc_histogram(const float *x, int64_t n, float lo, float hi, int32_t nbins, uint64_t *hist)
{
    float w = hi - lo;
    float inv_w = (w > 0.0f && w <= FLT_MAX) ? (float)nbins / w : 0.0f;
    float top = (float)(nbins - 1);
    for (int32_t b = 0; b < nbins; ++b) hist[b] = 0;
    for (int64_t i = 0; i < n; ++i) {
        float d = x[i] - lo;
        float t = d * inv_w;
        float f = floorf(t);
        if (!(f >= 0.0f)) f = 0.0f;      /* also catches NaN */
        if (f > top) f = top;
        hist[(int32_t)f] += 1;
    }
}

/* Sec. 6.3 Eq. 10-12: folding batch normalisation into the convolution before it.
 * Per output channel c: f_c = gamma_c / sqrt(var_c) (the paper's sqrt(sigma^2), no epsilon),
 * A = f_c * W, C = f_c * (B - mu_c) + beta_c.  fp32, one rounding per operation. */
void orc_bn_fold(const float *w, int64_t channels, int64_t inner, const float *gamma,
                 const float *var, const float *bias, const float *mean, const float *beta,
                 float *w_out, float *bias_out)
{
    for (int64_t c = 0; c < channels; ++c) {
        float root = sqrtf(var[c]);
        float f = gamma[c] / root;
        for (int64_t j = 0; j < inner; ++j) w_out[c * inner + j] = f * w[c * inner + j];
        if (bias_out) {
            float b = bias ? bias[c] : 0.0f;
            float d = b - mean[c];
            float p = f * d;
            bias_out[c] = p + beta[c];
        }
    }
}
