/*
 * Memory-safety exerciser of the CPU oracle (TEST INFRASTRUCTURE, like the oracle itself).
 * Built together with merit_oracle.c under -fsanitize=address,undefined and run by
 * tests/test_host_sanitized.py: every ref_ function on small shapes whose buffers are
 * malloc'ed to the exact size (so a read or write one element out of bounds is reported),
 * including the shapes where an index rule is most likely to slip: padding as large as the
 * window, strides larger than the window, windows larger than the image, frames the block
 * does not divide, one-pixel images.  Values are not judged here (the pins do that), only
 * a few exact facts that cost nothing.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double ref_half_to_double(uint16_t h);
uint16_t ref_double_to_half(double d);
int ref_conv2d(const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int, int, int, int, int, int);
int ref_conv2d_relu(const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int, int, int, int, int, int);
int ref_conv2d_dilated(const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int, int, int, int, int,
                       int, int, int, int);
int ref_conv2d_residual(const uint16_t *, const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int,
                        int, int, int, int, int, int);
int ref_conv2d_depthwise(const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int, int, int, int, int);
int ref_pool2d(const float *, float *, int, int, int, int, int, int, int, int, int, int, int);
int ref_sad_search(const uint8_t *, const uint8_t *, int32_t *, int32_t *, int, int, int, int);
int ref_sad_surface(const uint8_t *, const uint8_t *, int32_t *, int, int, int, int, int, int);
int ref_correlation(const uint16_t *, const uint16_t *, uint16_t *, int, int, int, int, int, int);
int ref_sepfilter(const float *, const float *, const float *, float *, int, int, int, int);
int ref_bilateral(const float *, const float *, const float *, float *, int, int, int, int, double);

static int failures = 0;
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "oracle_check: %s failed at line %d\n", #c, __LINE__); ++failures; } } while (0)

static uint64_t state = 1911;
static uint32_t rnd(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static uint16_t *halves(size_t n)
{
    uint16_t *p = malloc(n * 2 + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = ref_double_to_half(((int)(rnd() % 2001) - 1000) / 500.0);
    return p;
}
static float *floats(size_t n)
{
    float *p = malloc(n * 4 + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = (float)(((int)(rnd() % 2001) - 1000) / 100.0);
    return p;
}
static uint8_t *bytes(size_t n)
{
    uint8_t *p = malloc(n + (n == 0));
    for (size_t i = 0; i < n; ++i) p[i] = (uint8_t)rnd();
    return p;
}
static int ext(int I, int k, int s, int p, int d) { return (I + 2 * p - ((k - 1) * d + 1)) / s + 1; }

static void conv_case(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw, int ph, int pw, int dh,
                      int dw)
{
    const int OH = ext(H, kh, sh, ph, dh), OW = ext(W, kw, sw, pw, dw);
    if (OH <= 0 || OW <= 0) return;
    uint16_t *x = halves((size_t)N * Cin * H * W), *w = halves((size_t)Cout * Cin * kh * kw);
    const size_t ny = (size_t)N * Cout * OH * OW;
    uint16_t *y = malloc(ny * 2 + 1), *r = halves(ny);
    CHECK(ref_conv2d_dilated(x, w, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, 1) == 0);
    for (size_t i = 0; i < ny; ++i) CHECK(!(y[i] & 0x8000));                /* clipped: no sign bit */
    if (dh == 1 && dw == 1) {
        CHECK(ref_conv2d(x, w, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw) == 0);
        CHECK(ref_conv2d_relu(x, w, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw) == 0);
        CHECK(ref_conv2d_residual(x, w, r, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 0) == 0);
        if (Cin == Cout) {                                                    /* one kernel per channel */
            uint16_t *wd = halves((size_t)Cin * kh * kw);
            CHECK(ref_conv2d_depthwise(x, wd, y, N, Cin, H, W, kh, kw, sh, sw, ph, pw) == 0);
            free(wd);
        }
    }
    free(x); free(w); free(y); free(r);
}

static void pool_case(int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw)
{
    const int OH = ext(H, kh, sh, ph, 1), OW = ext(W, kw, sw, pw, 1);
    if (OH <= 0 || OW <= 0) return;
    const size_t nx = (size_t)N * C * H * W, ny = (size_t)N * C * OH * OW;
    float *x = floats(nx), *y = malloc(ny * 4 + 1);
    for (int avg = 0; avg < 2; ++avg) CHECK(ref_pool2d(x, y, N, C, H, W, kh, kw, sh, sw, ph, pw, avg) == 0);
    for (size_t i = 0; i < nx; ++i) x[i] = -2.5f;                             /* a constant stays that constant */
    CHECK(ref_pool2d(x, y, N, C, H, W, kh, kw, sh, sw, ph, pw, 1) == 0);
    for (size_t i = 0; i < ny; ++i) CHECK(y[i] == -2.5f || y[i] == 0.0f);     /* 0: a window with no element */
    free(x); free(y);
}

static void sad_case(int H, int W, int B, int R)
{
    const int nby = (H + B - 1) / B, nbx = (W + B - 1) / B, n = 2 * R + 1;
    uint8_t *cur = bytes((size_t)H * W), *ref = bytes((size_t)H * W);
    int32_t *sad = malloc((size_t)nby * nbx * 4), *mv = malloc((size_t)nby * nbx * 8);
    int32_t *surf = malloc((size_t)n * n * 4);
    CHECK(ref_sad_search(cur, ref, sad, mv, H, W, B, R) == 0);
    CHECK(ref_sad_surface(cur, ref, surf, H, W, B, R, nby - 1, nbx - 1) == 0);
    int32_t best = surf[0];
    for (int i = 1; i < n * n; ++i) if (surf[i] < best) best = surf[i];
    CHECK(best == sad[nby * nbx - 1]);
    CHECK(ref_sad_search(cur, cur, sad, mv, H, W, B, R) == 0);               /* a frame against itself */
    for (int i = 0; i < nby * nbx; ++i) CHECK(sad[i] == 0);
    free(cur); free(ref); free(sad); free(mv); free(surf);
}

int main(void)
{
    static const int conv[][13] = {
        /* N Cin H  W Cout kh kw sh sw ph pw dh dw */
        {1, 1, 1, 1, 1, 1, 1, 1, 1, 0, 0, 1, 1},   {2, 3, 7, 9, 4, 3, 3, 1, 1, 1, 1, 1, 1},
        {1, 2, 5, 5, 2, 3, 3, 2, 2, 3, 3, 1, 1},   {1, 3, 9, 8, 3, 7, 5, 4, 3, 3, 2, 1, 1},   /* padding = window, large strides */
        {1, 2, 4, 6, 2, 5, 7, 1, 1, 2, 3, 1, 1},   {1, 1, 11, 13, 2, 3, 3, 1, 2, 2, 4, 2, 3}, /* window > image; dilated */
        {0, 2, 4, 4, 2, 3, 3, 1, 1, 1, 1, 1, 1},   {1, 5, 3, 17, 5, 1, 11, 1, 4, 0, 5, 1, 1},
    };
    for (size_t i = 0; i < sizeof conv / sizeof conv[0]; ++i) {
        const int *c = conv[i];
        conv_case(c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8], c[9], c[10], c[11], c[12]);
    }
    static const int pool[][10] = {
        {1, 1, 1, 1, 1, 1, 1, 1, 0, 0}, {2, 3, 9, 7, 3, 3, 2, 2, 1, 1}, {1, 2, 16, 32, 3, 3, 2, 2, 3, 1},
        {1, 2, 6, 5, 3, 3, 2, 2, 3, 3}, {1, 1, 5, 6, 7, 8, 1, 1, 1, 1}, {1, 2, 10, 10, 2, 2, 5, 5, 0, 0},
        {3, 1, 7, 7, 7, 7, 1, 1, 0, 0}, {1, 1, 4, 4, 2, 2, 2, 2, 1, 1},
    };
    for (size_t i = 0; i < sizeof pool / sizeof pool[0]; ++i) {
        const int *c = pool[i];
        pool_case(c[0], c[1], c[2], c[3], c[4], c[5], c[6], c[7], c[8], c[9]);
    }
    sad_case(16, 16, 4, 2); sad_case(17, 33, 8, 4); sad_case(8, 8, 8, 9); sad_case(5, 40, 16, 3); sad_case(64, 64, 8, 4);

    {   /* correlation, separable and bilateral filters */
        static const int corr[][6] = {{1, 3, 5, 8, 2, 1}, {2, 9, 6, 7, 3, 2}, {1, 1, 1, 1, 4, 3}, {1, 16, 4, 16, 0, 1}};
        for (size_t i = 0; i < sizeof corr / sizeof corr[0]; ++i) {
            const int *c = corr[i];
            const int n = 2 * c[4] + 1;
            uint16_t *a = halves((size_t)c[0] * c[1] * c[2] * c[3]), *b = halves((size_t)c[0] * c[1] * c[2] * c[3]);
            uint16_t *y = malloc((size_t)c[0] * c[2] * c[3] * n * n * 2 + 1);
            CHECK(ref_correlation(a, b, y, c[0], c[1], c[2], c[3], c[4], c[5]) == 0);
            free(a); free(b); free(y);
        }
        static const int filt[][4] = {{1, 1, 1, 1}, {2, 7, 9, 3}, {1, 5, 4, 8}, {1, 3, 3, 31}, {1, 12, 10, 4}};
        for (size_t i = 0; i < sizeof filt / sizeof filt[0]; ++i) {
            const int *c = filt[i];
            const size_t n = (size_t)c[0] * c[1] * c[2];
            float *x = floats(n), *y = malloc(n * 4 + 1), *g1 = floats((size_t)c[3]), *g2 = floats((size_t)c[3]);
            for (int k = 0; k < c[3]; ++k) { g1[k] = fabsf(g1[k]) + 0.1f; g2[k] = fabsf(g2[k]) + 0.1f; }
            CHECK(ref_sepfilter(x, g1, g2, y, c[0], c[1], c[2], c[3]) == 0);
            CHECK(ref_bilateral(x, g1, g2, y, c[0], c[1], c[2], c[3], -0.05) == 0);
            float lo = x[0], hi = x[0];
            for (size_t j = 0; j < n; ++j) { if (x[j] < lo) lo = x[j]; if (x[j] > hi) hi = x[j]; }
            for (size_t j = 0; j < n; ++j) CHECK(y[j] >= lo && y[j] <= hi);   /* a weighted mean stays in range */
            free(x); free(y); free(g1); free(g2);
        }
    }
    /* binary16 conversions over every bit pattern: a round trip is the identity (NaNs aside) */
    for (uint32_t h = 0; h < 65536; ++h) {
        const double d = ref_half_to_double((uint16_t)h);
        if (d == d) CHECK(ref_double_to_half(d) == (uint16_t)h);
    }
    /* shapes the functions must refuse rather than index with */
    CHECK(ref_pool2d(NULL, NULL, 1, 0, 4, 4, 2, 2, 2, 2, 0, 0, 0) != 0);
    CHECK(ref_sepfilter(NULL, NULL, NULL, NULL, 1, 0, 4, 3) != 0);
    printf("oracle_check: %d failed checks\n", failures);
    return failures ? 1 : 0;
}
