/*
 * Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU oracle
 * (oracle/fq_oracle.c is compiled into this program with the sanitizers on).  It runs every
 * oracle function over small inputs chosen for their edges: extents of 0 and 1, ragged sizes, both
 * dtypes, non-finite values, one thread and several.  The arrays are heap blocks of exactly the
 * documented size, so any access outside them, and any undefined conversion or shift, stops the
 * program with a report.  Exit status 0: clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

float fqo_half_to_float(uint16_t h);
uint16_t fqo_float_to_half(float f);
void fqo_set_threads(int n);
void fqo_scale(const float *theta, int64_t C, float eps, float s_min, float s_max, float *s, uint8_t *clip_active);
void fqo_forward(const void *x, int dtype, int64_t outer, int64_t C, int64_t inner, const float *s, int32_t qmin,
                 int32_t qmax, void *y, int32_t *q);
void fqo_backward(const void *x, const void *gy, int dtype, int64_t outer, int64_t C, int64_t inner, const float *s,
                  const float *theta, const uint8_t *clip_active, int32_t qmin, int32_t qmax, void *gx, double *acc,
                  double *aabs, float *gs, float *gtheta);
void fqo_adam(const float *g, int64_t C, float lr, float beta1, float one_minus_beta1, float beta2,
              float one_minus_beta2, float eps, float bc1, float bc2, float *m, float *v, const float *theta_in,
              float *theta_out);
void fqo_distill(const void *a, const void *b, int dtype, int64_t N, int64_t C, int64_t M, double lambda, double eps,
                 double upstream, void *ga, double *out);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 32);
}
static float next_float(void) { return ((float)(next_u32() >> 8) / 8388608.0f - 1.0f) * 40.0f; }

/* exact-size heap block of n elements (at least one byte so that malloc(0) is not relied on) */
static void *block(size_t n, size_t esz) { return malloc(n * esz ? n * esz : 1); }

static void fill(void *p, int dtype, int64_t n, int specials)
{
    static const float odd[] = {0.0f, -0.0f, INFINITY, -INFINITY, NAN, 65504.0f, -65504.0f, 1e-8f, 127.5f, -128.5f};
    for (int64_t i = 0; i < n; ++i) {
        float v = (specials && i % 7 == 3) ? odd[(i / 7) % 10] : next_float();
        if (dtype == 0) ((uint16_t *)p)[i] = fqo_float_to_half(v);
        else ((float *)p)[i] = v;
    }
}

static void one_case(int dtype, int64_t outer, int64_t C, int64_t inner, int specials, int32_t qmin, int32_t qmax)
{
    const size_t esz = dtype == 0 ? 2 : 4;
    const int64_t n = outer * C * inner;
    void *x = block((size_t)n, esz), *gy = block((size_t)n, esz), *y = block((size_t)n, esz), *gx = block((size_t)n, esz);
    int32_t *q = block((size_t)n, 4);
    float *theta = block((size_t)C, 4), *s = block((size_t)C, 4), *gs = block((size_t)C, 4), *gt = block((size_t)C, 4);
    float *m = block((size_t)C, 4), *v = block((size_t)C, 4);
    uint8_t *active = block((size_t)C, 1);
    double *acc = block((size_t)C, 8), *aabs = block((size_t)C, 8);
    fill(x, dtype, n, specials);
    fill(gy, dtype, n, specials);
    for (int64_t c = 0; c < C; ++c) {
        theta[c] = (c % 5 == 4 && specials) ? 200.0f : -3.0f + 0.37f * (float)(c % 11);
        m[c] = 0.01f * (float)c;
        v[c] = 0.02f * (float)c;
    }
    fqo_scale(theta, C, 0.0f, specials ? 0.05f : 1.17549435e-38f, specials ? 3.0f : INFINITY, s, active);
    fqo_forward(x, dtype, outer, C, inner, s, qmin, qmax, y, q);
    fqo_forward(x, dtype, outer, C, inner, s, qmin, qmax, y, NULL);
    fqo_forward(x, dtype, outer, C, inner, s, qmin, qmax, NULL, q);
    fqo_backward(x, gy, dtype, outer, C, inner, s, theta, active, qmin, qmax, gx, acc, aabs, gs, gt);
    fqo_backward(x, gy, dtype, outer, C, inner, s, theta, NULL, qmin, qmax, NULL, acc, NULL, NULL, NULL);
    fqo_adam(gt, C, 1e-3f, 0.9f, 0.1f, 0.999f, 0.001f, 1e-8f, 0.1f, 0.001f, m, v, theta, theta);
    double out[3];
    fqo_distill(x, gy, dtype, outer, C, inner, 0.5, 1e-8, 1.0, gx, out);
    fqo_distill(x, gy, dtype, outer, C, inner, 0.0, 0.0, 2.0, NULL, out);
    free(x); free(gy); free(y); free(gx); free(q); free(theta); free(s); free(gs); free(gt); free(m); free(v);
    free(active); free(acc); free(aabs);
}

int main(void)
{
    /* every binary16 pattern through both conversions */
    for (uint32_t h = 0; h < 65536u; ++h) {
        float f = fqo_half_to_float((uint16_t)h);
        uint16_t back = fqo_float_to_half(f);
        if (!isnan(f) && back != (uint16_t)h) { printf("half round trip failed at %u\n", h); return 1; }
    }
    static const float edge[] = {65519.99f, 65520.0f, 1e30f, -1e30f, 5.9604645e-8f, 2.9802322e-8f, 2.98e-8f, 6.1e-5f, NAN};
    for (size_t i = 0; i < sizeof edge / sizeof edge[0]; ++i) (void)fqo_float_to_half(edge[i]);

    static const int64_t shapes[][3] = {{0, 3, 5}, {2, 0, 5}, {2, 3, 0}, {1, 1, 1}, {1, 1, 17}, {3, 5, 7}, {2, 9, 64},
                                        {1, 37, 129}, {4, 1, 1000}};
    for (int threads = 1; threads <= 5; threads += 2) {
        fqo_set_threads(threads);
        for (size_t k = 0; k < sizeof shapes / sizeof shapes[0]; ++k)
            for (int dtype = 0; dtype < 2; ++dtype)
                for (int specials = 0; specials < 2; ++specials) {
                    one_case(dtype, shapes[k][0], shapes[k][1], shapes[k][2], specials, -128, 127);
                    one_case(dtype, shapes[k][0], shapes[k][1], shapes[k][2], specials, -8, 7);
                    one_case(dtype, shapes[k][0], shapes[k][1], shapes[k][2], specials, -32768, 32768);
                }
    }
    printf("oracle sanitizer run clean\n");
    return 0;
}
