/*
 * CPU oracle for the MERIT ranged inner-product hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what
 * the HIP library must compute.  Nothing in the product path may call it: only
 * the test-suite, the smoke check and the benchmark's cpu_baseline leg do.  It
 * shares no code, header, table or helper with the HIP sources.
 *
 * Every operation here is an instance of the paper's row-wise reduction
 *     Vec(C) = R(M(A), M(B), (.))                         (Section III, Eq. 1)
 * where M(.) gathers, for output index p and accumulation index a, the input
 * element at x_i = sum_j delta(i,d_j) (k_j s_j + o_j), k=(p,a)  (Section III-C,
 * Eq. 5), and (.) is one of
 *     dot product  v1^T v2                                (Section III-B, Eq. 3)
 *     L1 distance  ||v1 - v2||_1                          (Section III-B, Eq. 4)
 *     max / mean over the window                          (pooling; the paper
 *         only names pooling as a max/min use, Table "isa"; the definition
 *         used is the usual one with padding excluded)
 * written out as nested loops over p then a, with no tiling, blocking, fusion
 * or reordering.  Floating point accumulates in double; integers in int32.
 *
 * Pins: tests/test_oracle_*.py check these functions against closed forms,
 * invariants, the literal Eq.-5 evaluator in merit_literal.py on tiny inputs,
 * and CPU library routines (none of them derived from this file).
 * Parity unpinned: none.
 */
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* IEEE-754 binary16 <-> double, written out bit by bit                     */
/* ------------------------------------------------------------------------ */

/* binary16 -> double is exact. */
double ref_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);              /* subnormal or zero */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

/* double -> binary16, round to nearest, ties to even; overflow -> inf. */
uint16_t ref_double_to_half(double d)
{
    uint16_t sign = (uint16_t)(signbit(d) ? 0x8000u : 0u);
    if (isnan(d)) return (uint16_t)(sign | 0x7e00u);
    double a = fabs(d);
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e);                           /* a = m * 2^e, m in [0.5,1) */
    int expo = e - 1;                              /* a = 1.xxx * 2^expo        */
    if (expo < -14) expo = -14;                    /* subnormal range: fixed ulp */
    /* ulp of the target at this exponent is 2^(expo-10); scale so ulp == 1.   */
    double scaled = ldexp(a, 10 - expo);           /* exact: power-of-two scale */
    double r = nearbyint(scaled);                  /* default mode = ties-even  */
    /* r is an integer in [0, 2048]. */
    long q = (long)r;
    if (q >= 2048) { q >>= 1; expo += 1; }        /* mantissa carried out      */
    if (expo > 15) return (uint16_t)(sign | 0x7c00u);
    if (q < 1024) {
        /* subnormal (expo == -14 and no implicit bit) or zero */
        return (uint16_t)(sign | (uint16_t)q);
    }
    return (uint16_t)(sign | (uint16_t)((expo + 15) << 10) | (uint16_t)(q - 1024));
}

/* ------------------------------------------------------------------------ */
/* 2-D convolution, fp16 in / fp16 out, double accumulate                    */
/* ------------------------------------------------------------------------ */
/*
 * y[n,co,oy,ox] = half( sum_{ci,ky,kx} x[n,ci,oy*sh+ky-ph, ox*sw+kx-pw] * w[co,ci,ky,kx] )
 * Index pattern of the strided-convolution example (Section III-C, Eq. 6): the
 * window index is added to the strided output index, the kernel is NOT
 * flipped, weights are indexed [p1,a1,a2,a3] = [co,ci,ky,kx].  Input
 * coordinates that fall outside the tensor contribute zero.
 * x: [N,Cin,H,W] binary16, w: [Cout,Cin,kh,kw] binary16, y: [N,Cout,OH,OW].
 * Returns 0, or -1 on a bad shape.
 */
static int conv2d_postloop(const uint16_t *x, const uint16_t *w, const uint16_t *res, uint16_t *y,
                           int N, int Cin, int H, int W, int Cout,
                           int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw, int relu)
{
    if (N < 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 ||
        sh <= 0 || sw <= 0 || ph < 0 || pw < 0 || dh <= 0 || dw <= 0) return -1;
    const int eh = (kh - 1) * dh + 1, ew = (kw - 1) * dw + 1;   /* extent of the dilated window */
    if (H + 2 * ph < eh || W + 2 * pw < ew) return -1;
    const int OH = (H + 2 * ph - eh) / sh + 1;
    const int OW = (W + 2 * pw - ew) / sw + 1;
    long nco;
#pragma omp parallel for schedule(static)
    for (nco = 0; nco < (long)N * Cout; ++nco) {
        const int n = (int)(nco / Cout), co = (int)(nco % Cout);
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                double acc = 0.0;
                for (int ci = 0; ci < Cin; ++ci)
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int iy = oy * sh + ky * dh - ph;
                            const int ix = ox * sw + kx * dw - pw;
                            if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                            const double xv = ref_half_to_double(
                                x[(((size_t)n * Cin + ci) * H + iy) * W + ix]);
                            const double wv = ref_half_to_double(
                                w[(((size_t)co * Cin + ci) * kh + ky) * kw + kx]);
                            acc += xv * wv;
                        }
                const size_t o = (((size_t)n * Cout + co) * OH + oy) * OW + ox;
                if (res) acc += ref_half_to_double(res[o]);  /* PostLoop: a loaded tensor added to act */
                if (relu && !(acc > 0.0)) acc = 0.0;       /* PostLoop: max(act, 0) */
                y[o] = ref_double_to_half(acc);
            }
    }
    return 0;
}

int ref_conv2d(const uint16_t *x, const uint16_t *w, uint16_t *y,
               int N, int Cin, int H, int W, int Cout,
               int kh, int kw, int sh, int sw, int ph, int pw)
{
    return conv2d_postloop(x, w, NULL, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, 0);
}

/*
 * The same ranged inner product with the second product function of Section
 * III-B, max(v1^T v2, 0) (the fused ReLU layer; Listing 1's PostLoop): the
 * double sum is clipped at zero, then rounded once to binary16.
 */
int ref_conv2d_relu(const uint16_t *x, const uint16_t *w, uint16_t *y,
                    int N, int Cin, int H, int W, int Cout,
                    int kh, int kw, int sh, int sw, int ph, int pw)
{
    return conv2d_postloop(x, w, NULL, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, 1);
}

/*
 * Dilated form (Section III-C, the example after Eq. 6: I[a1, p2 + 2 a2, p3 + 2 a3]):
 * window index ky moves dh input rows, kx moves dw input columns,
 *   x[n, ci, oy*sh + ky*dh - ph, ox*sw + kx*dw - pw];
 * output extent floor((I + 2 pad - ((k-1) d + 1)) / s) + 1.  relu != 0 selects the clipped
 * product function.
 */
int ref_conv2d_dilated(const uint16_t *x, const uint16_t *w, uint16_t *y,
                       int N, int Cin, int H, int W, int Cout,
                       int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw, int relu)
{
    return conv2d_postloop(x, w, NULL, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, dh, dw, relu);
}

/*
 * Residual layer (Section III-B, the remark after Listing 1: a second tensor loaded and
 * added to the accumulator in PostLoop): r has the output's shape [N,Cout,OH,OW],
 *   y = fp16( sum + r )            relu == 0
 *   y = fp16( max(sum + r, 0) )    relu != 0   (the addition precedes the clip, as it
 *                                               precedes the max in Listing 1's PostLoop)
 * The addition is made in double on the exact sum: one rounding in all.
 */
int ref_conv2d_residual(const uint16_t *x, const uint16_t *w, const uint16_t *r, uint16_t *y,
                        int N, int Cin, int H, int W, int Cout,
                        int kh, int kw, int sh, int sw, int ph, int pw, int relu)
{
    if (!r) return -1;
    return conv2d_postloop(x, w, r, y, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, relu);
}

/*
 * Depthwise convolution: every channel is convolved with its own kh x kw kernel
 * (the dot product over the window indices only; the channel index is parallel):
 *   y[n,c,oy,ox] = fp16( sum_{ky,kx} x[n,c,oy*sh+ky-ph,ox*sw+kx-pw] * w[c,ky,kx] ),
 * zeros outside the image.  x: [N,C,H,W], w: [C,kh,kw], y: [N,C,OH,OW], binary16;
 * double accumulation, one rounding.  Returns 0, or -1 on a bad shape.
 */
int ref_conv2d_depthwise(const uint16_t *x, const uint16_t *w, uint16_t *y,
                         int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw)
{
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0) return -1;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return -1;
    const int OH = (H + 2 * ph - kh) / sh + 1;
    const int OW = (W + 2 * pw - kw) / sw + 1;
    long nc;
#pragma omp parallel for schedule(static)
    for (nc = 0; nc < (long)N * C; ++nc) {
        const int c = (int)(nc % C);
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                double acc = 0.0;
                for (int ky = 0; ky < kh; ++ky)
                    for (int kx = 0; kx < kw; ++kx) {
                        const int iy = oy * sh + ky - ph;
                        const int ix = ox * sw + kx - pw;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        acc += ref_half_to_double(x[((size_t)nc * H + iy) * W + ix]) *
                               ref_half_to_double(w[((size_t)c * kh + ky) * kw + kx]);
                    }
                y[((size_t)nc * OH + oy) * OW + ox] = ref_double_to_half(acc);
            }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* 2-D pooling, fp32                                                         */
/* ------------------------------------------------------------------------ */
/*
 * Window of output (oy,ox): rows oy*sh-ph .. +kh-1, columns ox*sw-pw .. +kw-1;
 * only coordinates inside the tensor take part.
 *   is_avg == 0: maximum of the in-range elements (scan ky-major, replace on
 *                strict >, starting from -infinity);
 *   is_avg != 0: their sum divided by their count, summed and divided in
 *                double, rounded once to float.
 * A window with no in-range element gives -inf (max) or 0 (avg).
 */
int ref_pool2d(const float *x, float *y, int N, int C, int H, int W,
               int kh, int kw, int sh, int sw, int ph, int pw, int is_avg)
{
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 ||
        sh <= 0 || sw <= 0 || ph < 0 || pw < 0) return -1;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return -1;
    const int OH = (H + 2 * ph - kh) / sh + 1;
    const int OW = (W + 2 * pw - kw) / sw + 1;
    long nc;
#pragma omp parallel for schedule(static)
    for (nc = 0; nc < (long)N * C; ++nc) {
        const float *xp = x + (size_t)nc * H * W;
        float *yp = y + (size_t)nc * OH * OW;
        for (int oy = 0; oy < OH; ++oy)
            for (int ox = 0; ox < OW; ++ox) {
                float m = -INFINITY;
                double sum = 0.0;
                int cnt = 0;
                for (int ky = 0; ky < kh; ++ky)
                    for (int kx = 0; kx < kw; ++kx) {
                        const int iy = oy * sh + ky - ph;
                        const int ix = ox * sw + kx - pw;
                        if (iy < 0 || iy >= H || ix < 0 || ix >= W) continue;
                        const float v = xp[(size_t)iy * W + ix];
                        if (v > m) m = v;
                        sum += (double)v;
                        ++cnt;
                    }
                if (is_avg)
                    yp[(size_t)oy * OW + ox] = cnt ? (float)(sum / (double)cnt) : 0.0f;
                else
                    yp[(size_t)oy * OW + ox] = m;
            }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Block-matching motion estimation: SAD + min/argmin over the search range  */
/* ------------------------------------------------------------------------ */
static inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/*
 * One candidate: SAD(by,bx,dy,dx) = sum_{i,j<B} | cur[clamp(by*B+i), clamp(bx*B+j)]
 *                 - ref[clamp(by*B+i+dy, 0, H-1), clamp(bx*B+j+dx, 0, W-1)] |
 * The second tensor is displaced by the search indices exactly as in the
 * correlation-layer example (Section III-C, Eq. 8): ref coordinate = cur
 * coordinate + displacement.  Reads outside a frame are clamped to the nearest
 * edge pixel, in both frames: a frame whose height or width is not a multiple of
 * B has ceil(H/B) x ceil(W/B) blocks, and the last ones reach past the edge
 * (both frames extended by border replication, the same as padding them to a
 * multiple of B that way first).  For frames B divides, no current-frame read is
 * ever clamped.
 */
int32_t ref_sad_candidate(const uint8_t *cur, const uint8_t *ref, int H, int W, int B,
                          int by, int bx, int dy, int dx)
{
    int32_t sad = 0;
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < B; ++j) {
            const int cy = by * B + i, cx = bx * B + j;
            const int ry = clampi(cy + dy, 0, H - 1);
            const int rx = clampi(cx + dx, 0, W - 1);
            const int d = (int)cur[(size_t)clampi(cy, 0, H - 1) * W + clampi(cx, 0, W - 1)] -
                          (int)ref[(size_t)ry * W + rx];
            sad += d < 0 ? -d : d;
        }
    return sad;
}

/*
 * Full search.  For every block (by,bx) scan dy = -R..R (outer), dx = -R..R
 * (inner) and keep the first candidate with the strictly smallest SAD, i.e.
 * ties go to the lowest raster index (dy+R)*(2R+1) + (dx+R).  This is the
 * outer level of a two-level ranged inner product (Section III-B): the inner
 * loop accumulates |a-b| over the block, the outer post-loop keeps the min.
 * sad: [nby*nbx] int32, mv: [nby*nbx][2] int32 = (dy, dx).
 */
int ref_sad_search(const uint8_t *cur, const uint8_t *ref, int32_t *sad, int32_t *mv,
                   int H, int W, int B, int R)
{
    if (H <= 0 || W <= 0 || B <= 0 || R < 0) return -1;
    const int nby = (H + B - 1) / B, nbx = (W + B - 1) / B;
    long b;
#pragma omp parallel for schedule(static)
    for (b = 0; b < (long)nby * nbx; ++b) {
        const int by = (int)(b / nbx), bx = (int)(b % nbx);
        int32_t best = INT32_MAX;
        int bdy = 0, bdx = 0;
        for (int dy = -R; dy <= R; ++dy)
            for (int dx = -R; dx <= R; ++dx) {
                const int32_t s = ref_sad_candidate(cur, ref, H, W, B, by, bx, dy, dx);
                if (s < best) { best = s; bdy = dy; bdx = dx; }
            }
        sad[b] = best;
        mv[2 * b + 0] = bdy;
        mv[2 * b + 1] = bdx;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Correlation layer, fp16 in / fp16 out                                      */
/* ------------------------------------------------------------------------ */
/*
 * Section III-C, Eq. 8:  M(I1)[p1,p2,p3,p4,a1] = I1[a1,p1,p2],
 *                        M(I2)[p1,p2,p3,p4,a1] = I2[a1,p1+p3,p2+p4],
 * reduced over the channel index a1 with the dot product (Eq. 3).  Here the two
 * displacement indices run over n = 2R+1 values each, centred and with a
 * stride: displacement (p3 - R)*sd rows, (p4 - R)*sd columns; a second-tensor
 * coordinate outside the image contributes 0.  No normalisation by the channel
 * count.  x1, x2: [N,C,H,W] binary16; y: [N,H,W,n,n] binary16 (the index order
 * (p1,p2,p3,p4) of the equation).  Exact products, double accumulation, one
 * rounding.  Returns 0, or -1 on a bad shape.
 */
int ref_correlation(const uint16_t *x1, const uint16_t *x2, uint16_t *y,
                    int N, int C, int H, int W, int R, int sd)
{
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || R < 0 || sd <= 0) return -1;
    const int n = 2 * R + 1;
    long row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < (long)N * H; ++row) {
        const int b = (int)(row / H), p1 = (int)(row % H);
        for (int p2 = 0; p2 < W; ++p2)
            for (int p3 = 0; p3 < n; ++p3)
                for (int p4 = 0; p4 < n; ++p4) {
                    const int yy = p1 + (p3 - R) * sd, xx = p2 + (p4 - R) * sd;
                    double acc = 0.0;
                    if (yy >= 0 && yy < H && xx >= 0 && xx < W)
                        for (int c = 0; c < C; ++c)
                            acc += ref_half_to_double(x1[(((size_t)b * C + c) * H + p1) * W + p2]) *
                                   ref_half_to_double(x2[(((size_t)b * C + c) * H + yy) * W + xx]);
                    y[((((size_t)b * H + p1) * W + p2) * n + p3) * n + p4] = ref_double_to_half(acc);
                }
    }
    return 0;
}

/* All (2R+1)^2 candidate SADs of one block, raster order (dy-major). */
int ref_sad_surface(const uint8_t *cur, const uint8_t *ref, int32_t *surface,
                    int H, int W, int B, int R, int by, int bx)
{
    if (H <= 0 || W <= 0 || B <= 0 || R < 0) return -1;
    if (by < 0 || by >= (H + B - 1) / B || bx < 0 || bx >= (W + B - 1) / B) return -1;
    int k = 0;
    for (int dy = -R; dy <= R; ++dy)
        for (int dx = -R; dx <= R; ++dx)
            surface[k++] = ref_sad_candidate(cur, ref, H, W, B, by, bx, dy, dx);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Separable filter, fp32                                                     */
/* ------------------------------------------------------------------------ */
/*
 * Two 1-D ranged inner products in a row (dot product, Section III-B Eq. 3), the window
 * centred as in the bilateral-filter call of Section VI-A (offset -k/2 on the window index):
 *   t[n,p1,p2] = sum_{a2<k} kx[a2] * x[n, p1, p2 + a2 - k/2]
 *   y[n,p1,p2] = sum_{a1<k} ky[a1] * t[n, p1 + a1 - k/2, p2]
 * k/2 is the integer quotient (an even k reaches one tap further back than forward); the
 * kernels are not flipped; coordinates outside the image are clamped to the nearest edge
 * pixel.  x, y: [N,H,W] float; kx, ky: [k] float.  Accumulated in double without rounding t,
 * rounded once to float.  Returns 0, or -1 on a bad shape.
 */
int ref_sepfilter(const float *x, const float *kx, const float *ky, float *y, int N, int H, int W, int k)
{
    if (N < 0 || H <= 0 || W <= 0 || k <= 0) return -1;
    const int c = k / 2;
    long row;
#pragma omp parallel for schedule(static)
    for (row = 0; row < (long)N * H; ++row) {
        const int n = (int)(row / H), p1 = (int)(row % H);
        const float *img = x + (size_t)n * H * W;
        for (int p2 = 0; p2 < W; ++p2) {
            double acc = 0.0;
            for (int a1 = 0; a1 < k; ++a1) {
                const int yy = clampi(p1 + a1 - c, 0, H - 1);
                double t = 0.0;
                for (int a2 = 0; a2 < k; ++a2)
                    t += (double)kx[a2] * (double)img[(size_t)yy * W + clampi(p2 + a2 - c, 0, W - 1)];
                acc += (double)ky[a1] * t;
            }
            y[(size_t)row * W + p2] = (float)acc;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Bilateral filter, fp32                                                     */
/* ------------------------------------------------------------------------ */
/*
 * Section VI-A (Listings 2 and 3): every output pixel is a normalised weighted mean of the
 * k x k window around it (window offset -k/2 on both window indices, coordinates clamped to
 * the image).  A neighbour's weight is the product of a range factor, exp(norm * (its value -
 * the centre pixel's value)^2), and a spatial factor gy[a1] * gx[a2] taken from two lookup
 * tables of length k (precomputed Gaussians in the paper).  norm is the range constant handed
 * to the kernel as it stands (-1/(2 sigma_r^2) for a Gaussian range term).
 * Everything in double, rounded once to float.  Returns 0, or -1 on a bad shape.
 */
int ref_bilateral(const float *x, const float *gx, const float *gy, float *y, int N, int H, int W, int k,
                  double norm)
{
    if (N < 0 || H <= 0 || W <= 0 || k <= 0) return -1;
    const int half = k / 2;
    long pix;
#pragma omp parallel for schedule(static)
    for (pix = 0; pix < (long)N * H * W; ++pix) {
        const int p2 = (int)(pix % W), p1 = (int)((pix / W) % H);
        const float *img = x + (size_t)(pix / ((long)H * W)) * H * W;
        const double here = (double)img[(size_t)p1 * W + p2];
        double numer = 0.0, denom = 0.0;
        for (int a1 = 0; a1 < k; ++a1) {
            const float *line = img + (size_t)clampi(p1 + a1 - half, 0, H - 1) * W;
            for (int a2 = 0; a2 < k; ++a2) {
                const double there = (double)line[clampi(p2 + a2 - half, 0, W - 1)];
                const double spatial = (double)gy[a1] * (double)gx[a2];
                const double range = exp(norm * (there - here) * (there - here));
                numer += range * spatial * there;
                denom += range * spatial;
            }
        }
        y[pix] = (float)(numer / denom);
    }
    return 0;
}

/* Number of threads the parallel loops above will use. */
int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void ref_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
