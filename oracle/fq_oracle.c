/*
 * CPU oracle for learnable-scale fake quantization (quantize -> dequantize).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, one-element-at-a-time
 * definition that the GPU library is checked against.  It shares no code,
 * header, table or helper with the GPU path and must never be called from
 * the product path: only the test-suite, the smoke check and the CPU-baseline
 * leg of the benchmark may load it.
 *
 * What it computes (DPVO-QAT++, Sec. 3.2 "Geometry-Preserving QAT"):
 *   scale    s = clip(softplus(theta) + eps, s_min, s_max)        Eq. (3)-(4)
 *   forward  FQ(x, s) = s * round(clip(x / s, qmin, qmax))        Eq. (5)-(6)
 *   backward straight-through estimator: round() is treated as the identity
 *            when differentiating, every other operation is differentiated
 *            exactly (the LSQ gradient the paper cites next to Eq. (5)).
 *
 * Arithmetic: IEEE-754 binary32, round-to-nearest-even, no contraction, no
 * fast-math (see the build flags in oracle/build.py); softplus and sigmoid
 * are evaluated in binary64 and the scale is rounded to binary32 once
 * (Sec. 4.1.5: scale parameters are kept in FP32 even under FP16 autocast).
 * FP16 tensors are widened to binary32 exactly, processed in binary32 and
 * narrowed with round-to-nearest-even (Sec. 3.3, "Mixed precision").
 * The scale gradient is accumulated in binary64.
 *
 * Pins (tests that do not use this file to check itself) are in
 * tests/test_oracle_*.py.  Parity unpinned: the numeric values of eps,
 * s_min, s_max (the paper prints symbols only); they are parameters here.
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

enum { FQO_F16 = 0, FQO_F32 = 1 };

/*
 * Threads for fqo_forward / fqo_backward (default 1).  The work is split over channels only:
 * every element is computed exactly as with one thread, and every channel's sum is still formed
 * by one thread, sequentially, in the same element order, so the results do not depend on the
 * count.  Used by the benchmark's all-cores baseline; the tests run with one thread and check
 * once that more threads change nothing.
 */
static int fqo_threads = 1;
void fqo_set_threads(int n) { fqo_threads = n < 1 ? 1 : n; }
int fqo_get_threads(void) { return fqo_threads; }

/* ---- binary16 <-> binary32, written out from the IEEE-754 formats ------- */

/* Widen a binary16 bit pattern; every binary16 value is exact in binary32. */
float fqo_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    uint32_t expo = (uint32_t)(h >> 10) & 0x1fu;
    uint32_t frac = (uint32_t)h & 0x3ffu;
    float mag;
    if (expo == 0x1fu) {
        if (frac == 0) {
            mag = INFINITY;
        } else {
            /* keep NaN payload bits */
            uint32_t bits = (sign << 31) | 0x7f800000u | (frac << 13);
            float f;
            memcpy(&f, &bits, sizeof f);
            return f;
        }
    } else if (expo == 0) {
        mag = ldexpf((float)frac, -24);                /* subnormal: frac * 2^-24 */
    } else {
        mag = ldexpf((float)(frac | 0x400u), (int)expo - 25); /* 1.frac * 2^(e-15) */
    }
    return sign ? -mag : mag;
}

/* Narrow binary32 to binary16, round-to-nearest, ties to even. */
uint16_t fqo_float_to_half(float f)
{
    uint32_t bits;
    memcpy(&bits, &f, sizeof bits);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    if (isnan(f)) {
        uint16_t payload = (uint16_t)((bits >> 13) & 0x3ffu);
        return (uint16_t)(sign | 0x7c00u | payload | 0x200u);
    }
    float a = fabsf(f);
    if (a >= 65520.0f)                /* halfway between 65504 and 2^16 rounds up */
        return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0f)
        return sign;
    int e;
    (void)frexpf(a, &e);              /* a = m * 2^e, 0.5 <= m < 1  =>  2^(e-1) <= a */
    int unit_exp = (e - 1) - 10;      /* exponent of one ulp for a normal binary16 */
    if (unit_exp < -24)
        unit_exp = -24;               /* subnormal range: fixed ulp 2^-24 */
    /* a / ulp is exact (power-of-two scaling); rintf rounds ties to even */
    float n = rintf(ldexpf(a, -unit_exp));
    float r = ldexpf(n, unit_exp);    /* the rounded magnitude, exact in binary32 */
    /* re-encode r */
    if (r >= 65520.0f)
        return (uint16_t)(sign | 0x7c00u);
    if (r < ldexpf(1.0f, -14)) {      /* subnormal result (or zero) */
        uint16_t fr = (uint16_t)ldexpf(r, 24);
        return (uint16_t)(sign | fr);
    }
    (void)frexpf(r, &e);
    uint16_t be = (uint16_t)((e - 1) + 15);
    uint16_t fr = (uint16_t)(ldexpf(r, 10 - (e - 1)) - 1024.0f);
    return (uint16_t)(sign | (uint16_t)(be << 10) | fr);
}

static float load_elem(const void *p, int dtype, int64_t i)
{
    if (dtype == FQO_F16)
        return fqo_half_to_float(((const uint16_t *)p)[i]);
    return ((const float *)p)[i];
}

static void store_elem(void *p, int dtype, int64_t i, float v)
{
    if (dtype == FQO_F16)
        ((uint16_t *)p)[i] = fqo_float_to_half(v);
    else
        ((float *)p)[i] = v;
}

/* ---- Eq. (3)-(4): s = clip(softplus(theta) + eps, s_min, s_max) --------- */

static double softplus64(double t)
{
    /* log(1 + e^t) written so that neither branch overflows */
    return fmax(t, 0.0) + log1p(exp(-fabs(t)));
}

static double sigmoid64(double t)
{
    /* d softplus / d theta */
    if (t >= 0.0)
        return 1.0 / (1.0 + exp(-t));
    double e = exp(t);
    return e / (1.0 + e);
}

/*
 * theta[C] -> s[C]; clip_active[c] = 1 where the clamp of Eq. (3)-(4) changed
 * the value (the clamp then has zero derivative; at the bounds themselves the
 * gradient passes).
 */
void fqo_scale(const float *theta, int64_t C, float eps, float s_min, float s_max,
               float *s, uint8_t *clip_active)
{
    for (int64_t c = 0; c < C; ++c) {
        double u64 = softplus64((double)theta[c]) + (double)eps;
        float u = (float)u64;                      /* the one rounding to binary32 */
        float v = u;
        if (v < s_min) v = s_min;
        if (v > s_max) v = s_max;
        s[c] = v;
        if (clip_active)
            clip_active[c] = (uint8_t)!(u >= s_min && u <= s_max);
    }
}

/* ---- Eq. (5): y = s * round(clip(x / s, qmin, qmax)) --------------------- */

static float clipf(float v, float lo, float hi)
{
    /* comparisons are false for NaN, so NaN passes through unchanged */
    if (v < lo) return lo;
    if (v > hi) return hi;
    return v;
}

/*
 * x, y: [outer, C, inner] contiguous, dtype as given.  s: [C] binary32.
 * q (optional): the integer codes, 0 where x is NaN.
 */
void fqo_forward(const void *x, int dtype, int64_t outer, int64_t C, int64_t inner,
                 const float *s, int32_t qmin, int32_t qmax, void *y, int32_t *q)
{
    const float lo = (float)qmin, hi = (float)qmax;
#pragma omp parallel for schedule(static) num_threads(fqo_threads) if (fqo_threads > 1)
    for (int64_t c = 0; c < C; ++c)
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t k = 0; k < inner; ++k) {
                int64_t i = (o * C + c) * inner + k;
                float xf = load_elem(x, dtype, i);
                float v = xf / s[c];               /* correctly rounded quotient */
                float cl = clipf(v, lo, hi);       /* clip first ...             */
                float qf = rintf(cl);              /* ... then round, ties even  */
                float yf = qf * s[c];
                if (y) store_elem(y, dtype, i, yf);
                if (q) q[i] = isnan(qf) ? 0 : (int32_t)qf;
            }
}

/* ---- STE backward -------------------------------------------------------- */
/*
 * With round() differentiated as the identity:
 *   dy/dx = 1 where qmin <= x/s <= qmax (both ends inclusive), else 0
 *   dy/ds = round(x/s) - x/s inside the range, qmin below it, qmax above it
 * gx = gy where in range, else +0 (a select, so a NaN/Inf gy in a masked slot
 * still gives +0).  A NaN quotient is out of range for gx and poisons the
 * scale gradient of its channel.
 * acc[c]  = sum over the channel of gy * dy/ds  (binary64)
 * aabs[c] = sum of |gy * dy/ds| (conditioning of the sum; optional)
 * gs[c] = (float)acc[c];  gtheta[c] = acc[c] * sigmoid(theta[c]) unless the
 * scale clamp is active for that channel, then 0.
 */
void fqo_backward(const void *x, const void *gy, int dtype,
                  int64_t outer, int64_t C, int64_t inner,
                  const float *s, const float *theta, const uint8_t *clip_active,
                  int32_t qmin, int32_t qmax,
                  void *gx, double *acc, double *aabs, float *gs, float *gtheta)
{
    const float lo = (float)qmin, hi = (float)qmax;
    /* channel by channel; within a channel the terms are added in memory order (o, then k) */
#pragma omp parallel for schedule(static) num_threads(fqo_threads) if (fqo_threads > 1)
    for (int64_t c = 0; c < C; ++c) {
        double sum = 0.0, sum_abs = 0.0;
        for (int64_t o = 0; o < outer; ++o)
            for (int64_t k = 0; k < inner; ++k) {
                int64_t i = (o * C + c) * inner + k;
                float xf = load_elem(x, dtype, i);
                float g = load_elem(gy, dtype, i);
                float v = xf / s[c];
                int in_range = (v >= lo) && (v <= hi);
                float t;
                if (in_range)
                    t = rintf(v) - v;
                else if (v < lo)
                    t = lo;
                else if (v > hi)
                    t = hi;
                else
                    t = v;                         /* NaN */
                if (gx) {
                    if (in_range) {
                        /* bit copy of gy */
                        if (dtype == FQO_F16)
                            ((uint16_t *)gx)[i] = ((const uint16_t *)gy)[i];
                        else
                            memcpy((float *)gx + i, (const float *)gy + i, sizeof(float));
                    } else {
                        store_elem(gx, dtype, i, 0.0f);
                    }
                }
                double term = (double)g * (double)t;
                sum += term;
                sum_abs += fabs(term);
            }
        acc[c] = sum;
        if (aabs) aabs[c] = sum_abs;
    }
    for (int64_t c = 0; c < C; ++c) {
        if (gs) gs[c] = (float)acc[c];
        if (gtheta) {
            if (clip_active && clip_active[c])
                gtheta[c] = 0.0f;
            else
                gtheta[c] = (float)(acc[c] * sigmoid64((double)theta[c]));
        }
    }
}

/* ---- one Adam step on the scale parameters -------------------------------- */
/*
 * The paper trains only the scale parameters, with Adam (Sec. 3.2 "Training details"); it
 * prints no hyper-parameters, so they are arguments.  Kingma & Ba (2015), Algorithm 1, in
 * binary32, every operation rounded on its own, in the order written:
 *   m     <- beta1*m + (1-beta1)*g
 *   v     <- beta2*v + ((1-beta2)*g)*g
 *   theta <- theta - (lr * (m/bc1)) / (sqrt(v/bc2) + eps)
 * The six constants beta1, 1-beta1, beta2, 1-beta2, bc1 = 1-beta1^t, bc2 = 1-beta2^t are
 * evaluated by the caller from binary64 hyper-parameters and rounded to binary32 once each
 * (1-beta2 formed in binary32 from a binary32 beta2 would be off by 1e-5 relative).
 * A channel whose gradient is not finite is left untouched (m, v, theta keep their values):
 * the "isfinite guard" of Sec. 4.1.5.
 */
void fqo_adam(const float *g, int64_t C, float lr, float beta1, float one_minus_beta1, float beta2,
              float one_minus_beta2, float eps, float bc1, float bc2,
              float *m, float *v, const float *theta_in, float *theta_out)
{
    for (int64_t c = 0; c < C; ++c) {
        if (!isfinite(g[c])) {
            theta_out[c] = theta_in[c];
            continue;
        }
        float mm = beta1 * m[c] + one_minus_beta1 * g[c];
        float vv = beta2 * v[c] + (one_minus_beta2 * g[c]) * g[c];
        float mhat = mm / bc1, vhat = vv / bc2;
        m[c] = mm;
        v[c] = vv;
        theta_out[c] = theta_in[c] - (lr * mhat) / (sqrtf(vhat) + eps);
    }
}

/* ---- distillation loss between student and teacher feature maps ----------- */
/*
 * One (student, teacher) pair of Eq. (7):  L = MSE(a, b) + lambda * (1 - CosSim(a, b)),
 * a, b: [N, C, M] contiguous (M = H*W).  The paper prints neither lambda, nor the axis of the
 * cosine, nor how it is averaged; the reading taken (what patch matching needs, and what the
 * per-operator code `cosine_similarity(a, b, dim=1).mean()` computes):
 *   mse    = mean over all N*C*M elements of (a - b)^2
 *   cos_p  = sum_c a b / (max(||a_p||, eps) * max(||b_p||, eps))   for every position p = (n, m),
 *            norms over the channel axis
 *   cosim  = mean over the N*M positions of cos_p
 * out[0] = mse, out[1] = cosim, out[2] = L.  If ga != NULL it receives upstream * dL/da in the
 * tensors' dtype: 2(a-b)/(N*C*M) - lambda/(N*M) * d cos_p / d a, with
 * d cos_p / d a_c = b_c / (na' * nb') - [ ||a_p|| > eps ] * cos_p * a_c / ||a_p||^2
 * (a clamped norm is a constant).  All arithmetic in binary64.
 */
void fqo_distill(const void *a, const void *b, int dtype, int64_t N, int64_t C, int64_t M,
                 double lambda, double eps, double upstream, void *ga, double *out)
{
    /* the two means run over up to 10^8 terms: accumulate them in long double (64-bit significand
       on x86-64) so that the oracle's own summation error stays below 1e-13 relative */
    long double sum_sq = 0.0L, sum_cos = 0.0L;
    const double k1 = 2.0 / ((double)N * (double)C * (double)M);
    const double k2 = lambda / ((double)N * (double)M);
    for (int64_t n = 0; n < N; ++n)
        for (int64_t m = 0; m < M; ++m) {
            double dot = 0.0, na = 0.0, nb = 0.0;
            for (int64_t c = 0; c < C; ++c) {
                int64_t i = (n * C + c) * M + m;
                double av = (double)load_elem(a, dtype, i), bv = (double)load_elem(b, dtype, i);
                dot += av * bv;
                na += av * av;
                nb += bv * bv;
                sum_sq += (long double)((av - bv) * (av - bv));
            }
            double ra = sqrt(na), rb = sqrt(nb);
            double ca = ra < eps ? eps : ra, cb = rb < eps ? eps : rb;   /* a NaN norm stays NaN */
            double cosp = dot / (ca * cb);
            sum_cos += (long double)cosp;
            if (ga) {
                double self = ra > eps ? cosp / na : 0.0;
                for (int64_t c = 0; c < C; ++c) {
                    int64_t i = (n * C + c) * M + m;
                    double av = (double)load_elem(a, dtype, i), bv = (double)load_elem(b, dtype, i);
                    double dcos = bv / (ca * cb) - self * av;
                    double g = upstream * (k1 * (av - bv) - k2 * dcos);
                    store_elem(ga, dtype, i, (float)g);
                }
            }
        }
    out[0] = (double)(sum_sq / ((long double)N * (long double)C * (long double)M));
    out[1] = (double)(sum_cos / ((long double)N * (long double)M));
    out[2] = out[0] + lambda * (1.0 - out[1]);
}
