// 2-D max / average pooling for gfx950: one-operand ranged reduce.
//
// k = (n, c, oy, ox | ky, kx);  M(x)[p,a] = x[n, c, oy*sh + ky - ph, ox*sw + kx - pw]
// (transform of Section III-C, Eq. 5), reduced over a with max or mean.  Each
// workgroup stages the minimal covering sub-tensor of its output tile
// (Section IV-A, Eq. 9) in LDS with coalesced loads, resolves padding there
// (-inf for max, 0 and an analytic count for mean) and expands the windows
// from LDS, so HBM sees every input element about once.
#include "merit_internal.h"

#include <math.h>

namespace merit {

typedef float v4f __attribute__((ext_vector_type(4)));

// ---------------------------------------------------------------------------
// Generic tile kernel: any window / stride / padding, scalar accesses.
// ---------------------------------------------------------------------------
template <bool AVG>
__global__ __launch_bounds__(256) void merit_pool2d_tile(PoolParams p, const float *__restrict__ x,
                                                        float *__restrict__ y)
{
    extern __shared__ __align__(16) float lds[];
    const int tid = threadIdx.x;
    const uint32_t wg = blockIdx.x;
    const uint32_t per_plane = (uint32_t)(p.tiles_x * p.tiles_y);
    const uint32_t nc = wg / per_plane;
    const uint32_t t = wg - nc * per_plane;
    const int tyi = (int)(t / (uint32_t)p.tiles_x);
    const int txi = (int)(t - (uint32_t)tyi * p.tiles_x);
    const int oy0 = tyi * p.TH, ox0 = txi * p.TW;
    const int y0 = oy0 * p.sh - p.ph, x0 = ox0 * p.sw - p.pw;
    const float fill = AVG ? 0.0f : -INFINITY;
    const float *xp = x + (size_t)nc * p.H * p.W;

    const int nstage = p.RH * p.RW;
    for (int i = tid; i < nstage; i += 256) {
        const int r = (int)fdiv((uint32_t)i, p.div_rw);
        const int c = i - r * p.RW;
        const int gy = y0 + r, gx = x0 + c;
        float v = fill;
        if (gy >= 0 && gy < p.H && gx >= 0 && gx < p.W) v = xp[(size_t)gy * p.W + gx];
        lds[r * p.pitch + c] = v;
    }
    __syncthreads();

    float *yp = y + (size_t)nc * p.OH * p.OW;
    const int nout = p.TH * p.TW;
    for (int o = tid; o < nout; o += 256) {
        const int ty = (int)fdiv((uint32_t)o, p.div_tw);
        const int tx = o - ty * p.TW;
        const int oy = oy0 + ty, ox = ox0 + tx;
        if (oy >= p.OH || ox >= p.OW) continue;
        const float *w = lds + (ty * p.sh) * p.pitch + tx * p.sw;
        float acc = fill;
        for (int ky = 0; ky < p.kh; ++ky)
            for (int kx = 0; kx < p.kw; ++kx) {
                const float v = w[ky * p.pitch + kx];
                if (AVG) acc += v;
                else acc = (v > acc) ? v : acc;
            }
        if (AVG) {
            const int wy0 = oy * p.sh - p.ph, wx0 = ox * p.sw - p.pw;
            const int cy = min(wy0 + p.kh, p.H) - max(wy0, 0);
            const int cx = min(wx0 + p.kw, p.W) - max(wx0, 0);
            const int cnt = max(cy, 0) * max(cx, 0);
            acc = cnt > 0 ? acc / (float)cnt : 0.0f;
        }
        yp[(size_t)oy * p.OW + ox] = acc;
    }
}

// ---------------------------------------------------------------------------
// Row-strip kernel: a workgroup owns TH full output rows of one (n,c) plane.
// The input rows it needs are one contiguous span of the plane, copied to LDS
// with 16-byte loads; 4 fill columns on either side and fill rows above/below
// make the window scan branch-free.  Each thread produces four adjacent outputs
// and stores them as one float4.  Needs W % 4 == 0, OW % 4 == 0, PW <= 4 and
// (OW-1)*SW - PW + KW - 1 <= W + 3.
// ---------------------------------------------------------------------------
template <int KH, int KW, int SH, int SW, int PW, bool AVG>
__global__ __launch_bounds__(256) void merit_pool2d_rows(PoolParams p, const float *__restrict__ x,
                                                        float *__restrict__ y)
{
    extern __shared__ __align__(16) float lds[];
    const int tid = threadIdx.x;
    const uint32_t wg = blockIdx.x;
    const uint32_t nc = wg / (uint32_t)p.tiles_y;
    const int strip = (int)(wg - nc * (uint32_t)p.tiles_y);
    const int oy0 = strip * p.TH;
    const int nrows = min(p.TH, p.OH - oy0);
    const int y0 = oy0 * SH - p.ph;
    const int RH = (nrows - 1) * SH + KH;
    const int W4 = p.W >> 2;
    const int P4 = W4 + 2;                    // float4 per staged row: fill | data | fill
    const float fill = AVG ? 0.0f : -INFINITY;
    const float4 fill4 = make_float4(fill, fill, fill, fill);
    const float *xp = x + (size_t)nc * p.H * p.W;
    float4 *lds4 = reinterpret_cast<float4 *>(lds);

    const int nstage = RH * P4;
    for (int i = tid; i < nstage; i += 256) {
        const int r = (int)fdiv((uint32_t)i, p.div_p4);
        const int c4 = i - r * P4;
        const int gy = y0 + r;
        float4 v = fill4;
        if (c4 >= 1 && c4 <= W4 && gy >= 0 && gy < p.H)
            v = reinterpret_cast<const float4 *>(xp + (size_t)gy * p.W)[c4 - 1];
        lds4[i] = v;
    }
    __syncthreads();

    const int OW4 = p.OW >> 2;
    const int pitch = P4 * 4;
    float *yp = y + (size_t)nc * p.OH * p.OW;
    const int nout = nrows * OW4;
    for (int o = tid; o < nout; o += 256) {
        const int ty = (int)fdiv((uint32_t)o, p.div_ow4);
        const int q = o - ty * OW4;
        const int oy = oy0 + ty;
        // 16-byte aligned start of the span the four windows read: staged column of
        // input x = 4*q*SW - 4, so tap kx of output v sits at index 4 - PW + v*SW + kx.
        const float *base = reinterpret_cast<const float *>(
            __builtin_assume_aligned(lds + (ty * SH) * pitch + 4 * q * SW, 16));
        float acc[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[v] = fill;
#pragma unroll
        for (int ky = 0; ky < KH; ++ky) {
            const float *row = reinterpret_cast<const float *>(
                __builtin_assume_aligned(base + ky * pitch, 16));
            // the four windows touch floats [4-PW, 4-PW+SPAN) of the row: read the
            // covering 16-byte chunks
            constexpr int SPAN = 3 * SW + KW;
            constexpr int C0 = (4 - PW) / 4, C1 = (4 - PW + SPAN + 3) / 4;
            float t[(C1 - C0) * 4];
#pragma unroll
            for (int c = C0; c < C1; ++c) {
                const float4 f = reinterpret_cast<const float4 *>(row)[c];
                t[(c - C0) * 4 + 0] = f.x; t[(c - C0) * 4 + 1] = f.y;
                t[(c - C0) * 4 + 2] = f.z; t[(c - C0) * 4 + 3] = f.w;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int kx = 0; kx < KW; ++kx) {
                    const float val = t[(4 - PW) - C0 * 4 + v * SW + kx];
                    if (AVG) acc[v] += val;
                    else acc[v] = (val > acc[v]) ? val : acc[v];
                }
        }
        if (AVG) {
            const int wy0 = oy * SH - p.ph;
            const int cy = min(wy0 + KH, p.H) - max(wy0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int wx0 = (4 * q + v) * SW - PW;
                const int cx = min(wx0 + KW, p.W) - max(wx0, 0);
                const int cnt = max(cy, 0) * max(cx, 0);       // 0: the window lies in the padding
                acc[v] = cnt > 0 ? acc[v] / (float)cnt : 0.0f;
            }
        }
        reinterpret_cast<float4 *>(yp + (size_t)oy * p.OW)[q] = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
}

// ---------------------------------------------------------------------------
// Streaming kernel for the 3x3 / stride 2 / pad 1 window on planes up to 256
// columns wide (W % 4 == 0).  No LDS and no barrier: a group of 2^lg_shift lanes
// owns TH output rows of one plane, lane t holds the 16-byte column chunk t of
// every input row of the strip in registers (each input element is loaded by
// exactly one lane, all 2*TH+1 row loads are issued before the first use), and
// the one halo column a lane needs -- the last float of its left neighbour's
// chunk -- arrives with a DPP wave shift instead of through memory.  The window
// is separable: a row pass (3-tap max or sum giving the lane's two outputs) and
// a column pass over three row results.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float dpp_from_lane_below(float v, float fill)
{
    // lane i receives the value of lane i-1; lane 0 keeps `fill`
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(fill), __float_as_int(v), 0x138 /* wave_shr:1 */,
                                                      0xf, 0xf, false));
}

template <bool AVG, int TH>
__global__ __launch_bounds__(256) void merit_pool2d_stream_k3s2p1(PoolParams p, const float *__restrict__ x,
                                                                 float *__restrict__ y)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lg = 1 << p.lg_shift;
    const int t = lane & (lg - 1);                          // 16-byte column chunk
    const int item = (wave << (6 - p.lg_shift)) + (lane >> p.lg_shift);
    const int W4 = p.W >> 2;
    const bool live = item < p.items && t < W4;
    const int nc = live ? item / p.tiles_y : 0;
    const int strip = live ? item - nc * p.tiles_y : 0;
    const int oy0 = strip * TH;
    const float fill = AVG ? 0.0f : -INFINITY;
    const float *xp = x + (size_t)nc * p.H * p.W + 4 * t;

    // rows 2*oy0-1 .. 2*oy0+2*TH-1, all loads in flight together
    float4 v[2 * TH + 1];
#pragma unroll
    for (int r = 0; r < 2 * TH + 1; ++r) {
        const int gy = 2 * oy0 - 1 + r;
        v[r] = make_float4(fill, fill, fill, fill);
        if (live && gy >= 0 && gy < p.H) {
            // every input byte is used once: non-temporal loads keep it from displacing
            // useful lines in the caches (measured: ~20 % less time on a cold input)
            const v4f q = __builtin_nontemporal_load(reinterpret_cast<const v4f *>(xp + (size_t)gy * p.W));
            v[r] = make_float4(q.x, q.y, q.z, q.w);
        }
    }
    // row pass: outputs 2t and 2t+1 read columns {4t-1,4t,4t+1} and {4t+1,4t+2,4t+3}
    float h0[2 * TH + 1], h1[2 * TH + 1];
#pragma unroll
    for (int r = 0; r < 2 * TH + 1; ++r) {
        float left = dpp_from_lane_below(v[r].w, fill);
        if (t == 0) left = fill;                            // column -1 is padding
        if (AVG) {
            h0[r] = (left + v[r].x) + v[r].y;
            h1[r] = (v[r].y + v[r].z) + v[r].w;
        } else {
            h0[r] = fmaxf(fmaxf(left, v[r].x), v[r].y);
            h1[r] = fmaxf(fmaxf(v[r].y, v[r].z), v[r].w);
        }
    }
    // column pass and store
    float *yp = y + (size_t)nc * p.OH * p.OW + 2 * t;
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        const int oy = oy0 + i;
        float o0, o1;
        if (AVG) {
            o0 = (h0[2 * i] + h0[2 * i + 1]) + h0[2 * i + 2];
            o1 = (h1[2 * i] + h1[2 * i + 1]) + h1[2 * i + 2];
            const int wy0 = 2 * oy - 1;
            const int cy = min(wy0 + 3, p.H) - max(wy0, 0);
            const int cx0 = min(4 * t + 2, p.W) - max(4 * t - 1, 0);
            const int cx1 = min(4 * t + 4, p.W) - (4 * t + 1);
            o0 = o0 / (float)(cy * cx0);
            o1 = o1 / (float)(cy * cx1);
        } else {
            o0 = fmaxf(fmaxf(h0[2 * i], h0[2 * i + 1]), h0[2 * i + 2]);
            o1 = fmaxf(fmaxf(h1[2 * i], h1[2 * i + 1]), h1[2 * i + 2]);
        }
        if (live && oy < p.OH) *reinterpret_cast<float2 *>(yp + (size_t)oy * p.OW) = make_float2(o0, o1);
    }
}

// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// One output per plane (OH = OW = 1: global pooling, the window covers what it can reach of
// the plane): a group of 4 to 64 lanes per plane (about four window elements per lane: a 7x7 plane
// takes 16 lanes, four planes per wavefront), lanes stride over the in-range window elements, four
// loads in flight each, the partial results are folded with lane exchanges inside the group.
// No LDS, no barrier.  (A whole wavefront per 49-element plane: 65536 wavefronts of one load each,
// 11 us for 12.8 MB.)
// ---------------------------------------------------------------------------
template <bool AVG>
__global__ __launch_bounds__(256) void merit_pool2d_plane(PoolParams p, const float *__restrict__ x,
                                                         float *__restrict__ y)
{
    const int lane = threadIdx.x & 63;
    const int wave = (int)blockIdx.x * 4 + (int)(threadIdx.x >> 6);
    const int lpp = 64 >> p.lg_shift;                               // lanes per plane
    const int l = lane & (lpp - 1);
    const int plane = (wave << p.lg_shift) + (lane >> (6 - p.lg_shift));
    const bool live = plane < p.NC;
    const int y0 = max(-p.ph, 0), y1 = min(-p.ph + p.kh, p.H);      // in-range part of the window
    const int x0 = max(-p.pw, 0), x1 = min(-p.pw + p.kw, p.W);
    const int rw = max(x1 - x0, 0), cnt = live ? max(y1 - y0, 0) * rw : 0;
    const float *xp = x + (size_t)(live ? plane : 0) * p.H * p.W;
    const float fill = AVG ? 0.0f : -INFINITY;
    float acc = fill;
    for (int i0 = l; i0 < cnt; i0 += 4 * lpp) {
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = min(i0 + k * lpp, cnt - 1);
            const int r = i / rw;
            v[k] = xp[(size_t)(y0 + r) * p.W + x0 + (i - r * rw)];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float t = i0 + k * lpp < cnt ? v[k] : fill;
            if (AVG) acc += t;
            else acc = (t > acc) ? t : acc;
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        if (off < lpp) {
            const float o = __shfl_xor(acc, off);
            if (AVG) acc += o;
            else acc = (o > acc) ? o : acc;
        }
    }
    if (live && l == 0) y[plane] = AVG ? (cnt > 0 ? acc / (float)cnt : 0.0f) : acc;
}

// ---------------------------------------------------------------------------
// 3x3 / stride 2 window on any width (padding 0 or 1): a lane per output column, no LDS, no
// barrier.  A group of 16, 32 or 64 lanes (the smallest that holds a row of outputs, 64-column
// chunks beyond that) owns LANES_TH output rows of one plane: per input row a lane loads its
// three columns (neighbouring lanes' loads overlap in one column and coalesce), reduces them,
// and every row result is used by the one or two output rows it belongs to.  All loads of a
// strip are issued before the first use.  tiles_x = column chunks, tiles_y = row strips.
// ---------------------------------------------------------------------------
constexpr int LANES_TH = 4;

template <bool AVG>
__global__ __launch_bounds__(256) void merit_pool2d_lanes_k3s2(PoolParams p, const float *__restrict__ x,
                                                              float *__restrict__ y)
{
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lpi = 64 >> p.lg_shift;                        // lanes per item
    const int l = lane & (lpi - 1);
    const int item = (wave << p.lg_shift) + (lane >> (6 - p.lg_shift));
    const bool live_item = item < p.items;
    const int it = live_item ? item : 0;
    const uint32_t q0 = fdiv((uint32_t)it, p.div_tiles_x);
    const int chunk = it - (int)q0 * p.tiles_x;
    const uint32_t nc = fdiv(q0, p.div_tiles_y);
    const int strip = (int)q0 - (int)nc * p.tiles_y;
    const int ox = chunk * 64 + l;
    const bool live = live_item && ox < p.OW;
    const int oy0 = strip * LANES_TH;
    const int ytop = oy0 * 2 - p.ph, xleft = min(ox, p.OW - 1) * 2 - p.pw;
    const float fill = AVG ? 0.0f : -INFINITY;
    const float *xp = x + (size_t)nc * p.H * p.W;

    float v[2 * LANES_TH + 1][3];
#pragma unroll
    for (int r = 0; r < 2 * LANES_TH + 1; ++r) {
        const int gy = ytop + r;
        const bool rowok = gy >= 0 && gy < p.H;
        const float *row = xp + (size_t)(rowok ? gy : 0) * p.W;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int gx = xleft + k;
            const bool ok = rowok && gx >= 0 && gx < p.W;
            const float t = row[ok ? gx : 0];                       // branch-free; replaced below
            v[r][k] = ok ? t : fill;
        }
    }
    float rr[2 * LANES_TH + 1];
#pragma unroll
    for (int r = 0; r < 2 * LANES_TH + 1; ++r)
        rr[r] = AVG ? (v[r][0] + v[r][1]) + v[r][2] : fmaxf(fmaxf(v[r][0], v[r][1]), v[r][2]);
    float *yp = y + (size_t)nc * p.OH * p.OW;
#pragma unroll
    for (int i = 0; i < LANES_TH; ++i) {
        const int oy = oy0 + i;
        float o = AVG ? (rr[2 * i] + rr[2 * i + 1]) + rr[2 * i + 2]
                      : fmaxf(fmaxf(rr[2 * i], rr[2 * i + 1]), rr[2 * i + 2]);
        if (AVG) {
            const int wy0 = 2 * oy - p.ph, wx0 = 2 * ox - p.pw;
            const int cy = min(wy0 + 3, p.H) - max(wy0, 0);
            const int cx = min(wx0 + 3, p.W) - max(wx0, 0);
            const int cnt = max(cy, 0) * max(cx, 0);
            o = cnt > 0 ? o / (float)cnt : 0.0f;
        }
        if (live && oy < p.OH) yp[(size_t)oy * p.OW + ox] = o;
    }
}

// ---------------------------------------------------------------------------
// Stride-2 windows on any width of 8 and more -- 3x3 with padding 0 or 1 (K = 3), 2x2 without padding
// (K = 2): a lane per TWO adjacent output columns, whose input columns 4j - pw .. 4j - pw + 3 are one
// 16-byte load per input row (fp32 rows start on any 4-byte boundary, which is all a 16-byte global
// load needs; K = 3 adds a 4-byte load for the fifth column) instead of six 4-byte loads.  The
// 16-byte load is moved inside the row where the lane's columns cross an edge (start clamped to
// [0, W - 4]) and the lane's columns are picked out of it by the distance d it was moved (-1 at the
// left edge with padding, 1..3 at the right edge; a column that is not among the four is outside the
// row: fill).  d and the validity of the fifth column are the same for every row of the strip.
// A group of 4, 8, 16, 32 or 64 lanes (the smallest that holds a row of outputs, 128-column chunks
// beyond that) owns LANES_TH output rows of one plane.  The same for 3x3 windows at stride 1 (S = 1).  No LDS, no barrier; all loads of a strip are
// issued before the first use.
// ---------------------------------------------------------------------------
typedef float float4u __attribute__((ext_vector_type(4), aligned(4)));

template <bool AVG, int K, int S = 2>
__global__ __launch_bounds__(256) void merit_pool2d_lanes2_s2(PoolParams p, const float *__restrict__ x,
                                                             float *__restrict__ y)
{
    // S = 1 (3x3 windows, padding 0 or 1; any width of 4 and more): the two outputs' columns ox - pw ..
    // ox - pw + 3 are the 16-byte load alone; 8 output rows per group from 10 input rows
    static_assert(S == 2 || K == 3, "stride 1: 3x3 windows");
    constexpr int TH = S == 1 ? 8 : LANES_TH;
    constexpr int ROWS = S == 1 ? TH + 2 : (K == 3 ? 2 * TH + 1 : 2 * TH);
    constexpr bool FIFTH = K == 3 && S == 2;
    const int lane = threadIdx.x & 63;
    const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lpi = 64 >> p.lg_shift;                        // lanes per item
    const int l = lane & (lpi - 1);
    const int item = (wave << p.lg_shift) + (lane >> (6 - p.lg_shift));
    const bool live_item = item < p.items;
    const int it = live_item ? item : 0;
    const uint32_t q0 = fdiv((uint32_t)it, p.div_tiles_x);
    const int chunk = it - (int)q0 * p.tiles_x;
    const uint32_t nc = fdiv(q0, p.div_tiles_y);
    const int strip = (int)q0 - (int)nc * p.tiles_y;
    const int ox = chunk * 128 + 2 * l;                      // the lane's first output column
    const int oy0 = strip * TH;
    const int ytop = oy0 * S - p.ph;
    const int c0 = min(S * ox - p.pw, p.W);                  // first of the lane's input columns (>= -1)
    const int s0 = min(max(c0, 0), p.W - 4);                 // start of the 16-byte load, inside the row
    const int d = c0 - s0;                                   // -1 .. 4
    const int c4 = c0 + 4;
    const bool ok4 = c4 < p.W;
    const int s4 = min(c4, p.W - 1);
    const float fill = AVG ? 0.0f : -INFINITY;
    const float *xp = x + (size_t)nc * p.H * p.W;

    float4u a[ROWS];
    float e[FIFTH ? ROWS : 1];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int gy = ytop + r;
        const bool rowok = gy >= 0 && gy < p.H;
        const float *row = xp + (size_t)(rowok ? gy : 0) * p.W;
        a[r] = *reinterpret_cast<const float4u *>(row + s0);
        if constexpr (FIFTH) e[r] = row[s4];
    }
    float ra[ROWS], rb[ROWS];
#pragma unroll
    for (int r = 0; r < ROWS; ++r) {
        const int gy = ytop + r;
        const bool rowok = gy >= 0 && gy < p.H;
        float v[5];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int k = i + d;
            const float t = k == 0 ? a[r].x : (k == 1 ? a[r].y : (k == 2 ? a[r].z : a[r].w));
            v[i] = (rowok && k >= 0 && k <= 3) ? t : fill;
        }
        if constexpr (FIFTH) {
            v[4] = (rowok && ok4) ? e[r] : fill;
            ra[r] = AVG ? (v[0] + v[1]) + v[2] : fmaxf(fmaxf(v[0], v[1]), v[2]);
            rb[r] = AVG ? (v[2] + v[3]) + v[4] : fmaxf(fmaxf(v[2], v[3]), v[4]);
        } else if constexpr (S == 1) {
            ra[r] = AVG ? (v[0] + v[1]) + v[2] : fmaxf(fmaxf(v[0], v[1]), v[2]);
            rb[r] = AVG ? (v[1] + v[2]) + v[3] : fmaxf(fmaxf(v[1], v[2]), v[3]);
        } else {
            ra[r] = AVG ? v[0] + v[1] : fmaxf(v[0], v[1]);
            rb[r] = AVG ? v[2] + v[3] : fmaxf(v[2], v[3]);
        }
    }
    float *yp = y + (size_t)nc * p.OH * p.OW;
#pragma unroll
    for (int i = 0; i < TH; ++i) {
        const int oy = oy0 + i;
        const int r0 = S * i;
        float oa, ob;
        if constexpr (K == 3) {
            oa = AVG ? (ra[r0] + ra[r0 + 1]) + ra[r0 + 2] : fmaxf(fmaxf(ra[r0], ra[r0 + 1]), ra[r0 + 2]);
            ob = AVG ? (rb[r0] + rb[r0 + 1]) + rb[r0 + 2] : fmaxf(fmaxf(rb[r0], rb[r0 + 1]), rb[r0 + 2]);
        } else {
            oa = AVG ? ra[r0] + ra[r0 + 1] : fmaxf(ra[r0], ra[r0 + 1]);
            ob = AVG ? rb[r0] + rb[r0 + 1] : fmaxf(rb[r0], rb[r0 + 1]);
        }
        if (AVG) {
            const int wy0 = S * oy - p.ph;
            const int cy = max(min(wy0 + K, p.H) - max(wy0, 0), 0);
            const int xa = S * ox - p.pw, xb = xa + S;
            const int ca = cy * max(min(xa + K, p.W) - max(xa, 0), 0);
            const int cb = cy * max(min(xb + K, p.W) - max(xb, 0), 0);
            oa = ca > 0 ? oa / (float)ca : 0.0f;
            ob = cb > 0 ? ob / (float)cb : 0.0f;
        }
        if (live_item && oy < p.OH) {
            if (ox < p.OW) yp[(size_t)oy * p.OW + ox] = oa;
            if (ox + 1 < p.OW) yp[(size_t)oy * p.OW + ox + 1] = ob;
        }
    }
}

template <typename K>
static hipError_t launch(K kernel, const PoolParams &p, const float *x, float *y, hipStream_t s,
                         size_t lds_bytes, uint32_t grid)
{
    if (grid == 0) return hipSuccess;
    if (lds_bytes > 64 * 1024) {       // wide rows: more dynamic LDS than a kernel gets by default
        static std::atomic<int> raised{0};                  // (one per kernel instance: K is its type)
        if (hipError_t e = raise_lds_limit_once(reinterpret_cast<const void *>(kernel), raised); e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), lds_bytes, s, p, x, y);
    return hipGetLastError();
}

hipError_t launch_pool2d(const PoolParams &p, const float *x, float *y, hipStream_t s)
{
    const uint32_t grid = (uint32_t)p.grid;
    const size_t lds_bytes = (size_t)p.RH * p.pitch * sizeof(float);
    switch (p.variant) {
    case POOL_LANES_K3S2:
        return p.is_avg ? launch(merit_pool2d_lanes_k3s2<true>, p, x, y, s, 0, grid)
                        : launch(merit_pool2d_lanes_k3s2<false>, p, x, y, s, 0, grid);
    case POOL_LANES2_K3S2:
        if (p.sh == 1)
            return p.is_avg ? launch(merit_pool2d_lanes2_s2<true, 3, 1>, p, x, y, s, 0, grid)
                            : launch(merit_pool2d_lanes2_s2<false, 3, 1>, p, x, y, s, 0, grid);
        if (p.kh == 2)
            return p.is_avg ? launch(merit_pool2d_lanes2_s2<true, 2>, p, x, y, s, 0, grid)
                            : launch(merit_pool2d_lanes2_s2<false, 2>, p, x, y, s, 0, grid);
        return p.is_avg ? launch(merit_pool2d_lanes2_s2<true, 3>, p, x, y, s, 0, grid)
                        : launch(merit_pool2d_lanes2_s2<false, 3>, p, x, y, s, 0, grid);
    case POOL_PLANE:
        return p.is_avg ? launch(merit_pool2d_plane<true>, p, x, y, s, 0, grid)
                        : launch(merit_pool2d_plane<false>, p, x, y, s, 0, grid);
    case POOL_STREAM_K3S2P1:
        if (p.TH == 4)
            return p.is_avg ? launch(merit_pool2d_stream_k3s2p1<true, 4>, p, x, y, s, 0, grid)
                            : launch(merit_pool2d_stream_k3s2p1<false, 4>, p, x, y, s, 0, grid);
        if (p.TH == 7)
            return p.is_avg ? launch(merit_pool2d_stream_k3s2p1<true, 7>, p, x, y, s, 0, grid)
                            : launch(merit_pool2d_stream_k3s2p1<false, 7>, p, x, y, s, 0, grid);
        return p.is_avg ? launch(merit_pool2d_stream_k3s2p1<true, 8>, p, x, y, s, 0, grid)
                        : launch(merit_pool2d_stream_k3s2p1<false, 8>, p, x, y, s, 0, grid);
    case POOL_ROWS_K3S2P1:
        return p.is_avg ? launch(merit_pool2d_rows<3, 3, 2, 2, 1, true>, p, x, y, s, lds_bytes, grid)
                        : launch(merit_pool2d_rows<3, 3, 2, 2, 1, false>, p, x, y, s, lds_bytes, grid);
    case POOL_ROWS_K2S2P0:
        return p.is_avg ? launch(merit_pool2d_rows<2, 2, 2, 2, 0, true>, p, x, y, s, lds_bytes, grid)
                        : launch(merit_pool2d_rows<2, 2, 2, 2, 0, false>, p, x, y, s, lds_bytes, grid);
    case POOL_ROWS_K3S1P1:
        return p.is_avg ? launch(merit_pool2d_rows<3, 3, 1, 1, 1, true>, p, x, y, s, lds_bytes, grid)
                        : launch(merit_pool2d_rows<3, 3, 1, 1, 1, false>, p, x, y, s, lds_bytes, grid);
    default:
        return p.is_avg ? launch(merit_pool2d_tile<true>, p, x, y, s, lds_bytes, grid)
                        : launch(merit_pool2d_tile<false>, p, x, y, s, lds_bytes, grid);
    }
}

const char *pool_kernel_name(const PoolParams &p)
{
    switch (p.variant) {
    case POOL_PLANE: return p.is_avg ? "merit_pool2d_plane<avg>" : "merit_pool2d_plane<max>";
    case POOL_LANES_K3S2: return p.is_avg ? "merit_pool2d_lanes_k3s2<avg>" : "merit_pool2d_lanes_k3s2<max>";
    case POOL_LANES2_K3S2:
        if (p.sh == 1) return p.is_avg ? "merit_pool2d_lanes2_s2<avg,3,1>" : "merit_pool2d_lanes2_s2<max,3,1>";
        if (p.kh == 2) return p.is_avg ? "merit_pool2d_lanes2_s2<avg,2>" : "merit_pool2d_lanes2_s2<max,2>";
        return p.is_avg ? "merit_pool2d_lanes2_s2<avg,3>" : "merit_pool2d_lanes2_s2<max,3>";
    case POOL_STREAM_K3S2P1: return p.is_avg ? "merit_pool2d_stream_k3s2p1<avg>" : "merit_pool2d_stream_k3s2p1<max>";
    case POOL_ROWS_K3S2P1: return p.is_avg ? "merit_pool2d_rows<3,3,2,2,1,avg>" : "merit_pool2d_rows<3,3,2,2,1,max>";
    case POOL_ROWS_K2S2P0: return p.is_avg ? "merit_pool2d_rows<2,2,2,2,0,avg>" : "merit_pool2d_rows<2,2,2,2,0,max>";
    case POOL_ROWS_K3S1P1: return p.is_avg ? "merit_pool2d_rows<3,3,1,1,1,avg>" : "merit_pool2d_rows<3,3,1,1,1,max>";
    default: return p.is_avg ? "merit_pool2d_tile<avg>" : "merit_pool2d_tile<max>";
    }
}

}  // namespace merit
