// Bilateral filter for gfx950 (Section VI-A, Listings 2 and 3): every output pixel is the
// normalised weighted mean of its k x k window (window offset -k/2 on both window indices); a
// neighbour's weight is exp(norm * (its difference to the centre pixel)^2) times one entry
// of each of two spatial lookup tables of length k,
// with coordinates clamped to the image.  k*k exponentials per pixel against 8 bytes of memory
// traffic: bound by the vector ALU (v_exp_f32 runs at a quarter of the plain rate).
//
// A workgroup owns 16 x 64 output pixels (the listing's 16-row tiles, a wavefront wide); the
// covering sub-tensor (Section IV-A, Eq. 9) is staged in LDS with the clamping resolved
// there, from column x0 - c4 (k/2 rounded up to 4), so that for W % 4 == 0 the staging is
// aligned 16-byte loads without a branch.  A thread makes four outputs of one column, four
// rows apart: lanes run along the row (conflict-free 4-byte LDS reads) and the four
// independent chains hide the latency of the exponential.  Five vector instructions per tap:
// with s = sqrt(|norm| log2 e), the scaled difference d' = center*s - v*s is one fused
// multiply-add, the weight exp(d*d*norm) * gx[a2] = 2^(-+ d'*d' + log2 gx[a2]) one more and
// the base-2 exponential, then wsum += w and wxsum += w*v; gy[a1] is applied once per window
// row to the row's partial sums.  (A spatial table entry of 0 gives log2 = -inf and weight 0.)
#include "merit_internal.h"

namespace merit {

typedef float float4v __attribute__((ext_vector_type(4)));

// Staging of the covering sub-tensor: every element is a real (clamped) pixel.
__device__ __forceinline__ void stage_clamped(const BilatParams &p, const float *__restrict__ img, float *in, int x0,
                                              int y0, int RH, int tid)
{
    if ((p.W & 3) == 0) {
        constexpr int SB = 4;
        const int P4 = p.PI >> 2, W4 = p.W >> 2;
        const int g0 = (x0 - p.c4) >> 2;                  // first staged 4-column group (may be < 0)
        const int total = RH * P4;
        for (int e0 = tid; e0 < total; e0 += 256 * SB) {
            float4v v[SB];
            int g4[SB];
#pragma unroll
            for (int b = 0; b < SB; ++b) {
                const int e = min(e0 + 256 * b, total - 1);
                const int r = (int)fdiv((uint32_t)e, p.div_p4);
                g4[b] = g0 + (e - r * P4);
                const int gyy = min(max(y0 - p.c + r, 0), p.H - 1);
                v[b] = *reinterpret_cast<const float4v *>(img + (size_t)gyy * p.W + 4 * min(max(g4[b], 0), W4 - 1));
            }
#pragma unroll
            for (int b = 0; b < SB; ++b) {
                const bool inside = g4[b] >= 0 && g4[b] < W4;       // else: four copies of the edge pixel
                const float edge = g4[b] < 0 ? v[b].x : v[b].w;
                float4v o;
                o.x = inside ? v[b].x : edge; o.y = inside ? v[b].y : edge;
                o.z = inside ? v[b].z : edge; o.w = inside ? v[b].w : edge;
                if (e0 + 256 * b < total) reinterpret_cast<float4v *>(in)[e0 + 256 * b] = o;
            }
        }
    } else {
        const int total = RH * p.PI;
        for (int e = tid; e < total; e += 256) {
            const int r = e / p.PI;
            const int cc = e - r * p.PI;
            const int gyy = min(max(y0 - p.c + r, 0), p.H - 1);
            const int gxx = min(max(x0 - p.c4 + cc, 0), p.W - 1);
            in[e] = img[(size_t)gyy * p.W + gxx];
        }
    }
}

// NEG: the range constant is <= 0 (the usual decaying range term)
template <bool NEG>
__global__ __launch_bounds__(256) void merit_bilateral_tile(BilatParams p, const float *__restrict__ x,
                                                           const float *__restrict__ gx,
                                                           const float *__restrict__ gy, float *__restrict__ y)
{
    constexpr int TH = 16, TW = 64;
    extern __shared__ __align__(16) float smem[];
    const int RH = TH + p.k - 1;                          // staged rows
    float *in = smem;                                     // [RH][PI]
    float *wxl = in + RH * p.PI;                          // [k]
    float *wyl = wxl + p.k;                               // [k]

    const int tid = threadIdx.x;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: every XCD takes a
    // contiguous run of the raster-ordered tile list (a band of tile rows), so the halo rows and
    // the cache lines two neighbouring tiles share are fetched by one L2 once.  (With tile
    // blockIdx.x itself every neighbour sat on another XCD and the image was fetched 2.95 times.)
    const uint32_t g = xcd_band_item(blockIdx.x, (int)(gridDim.x >> 3), (int)(gridDim.x & 7));
    const uint32_t q0 = fdiv(g, p.div_tiles_x);
    const int tx = (int)(g - q0 * (uint32_t)p.tiles_x);
    const int n = (int)fdiv(q0, p.div_tiles_y);
    const int ty = (int)(q0 - (uint32_t)n * (uint32_t)p.tiles_y);
    const int x0 = tx * TW, y0 = ty * TH;
    const float *img = x + (size_t)n * p.H * p.W;

    if (tid < p.k) {
        wxl[tid] = __builtin_amdgcn_logf(gx[tid]);        // log2
        wyl[tid] = gy[tid];
    }
    stage_clamped(p, img, in, x0, y0, RH, tid);
    __syncthreads();

    // outputs (row0 + 4j, col), j < 4; staged column of tap a2 for output column col:
    // col + a2 - c + c4
    const int col = tid & 63, row0 = tid >> 6;
    const int dcol = col + p.c4 - p.c;
    float cen[4], wsum[4], wxsum[4];                      // cen: centre pixel times s
    const float sc = p.scale;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        cen[j] = in[(row0 + 4 * j + p.c) * p.PI + dcol + p.c] * sc;
        wsum[j] = 0.0f;
        wxsum[j] = 0.0f;
    }
    for (int a1 = 0; a1 < p.k; ++a1) {
        const float gyv = wyl[a1];
        const float *rowp = in + (row0 + a1) * p.PI + dcol;
        float rs[4] = {0.0f, 0.0f, 0.0f, 0.0f}, rxs[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 2
        for (int a2 = 0; a2 < p.k; ++a2) {
            const float lgx = wxl[a2];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = rowp[4 * j * p.PI + a2];
                const float d = fmaf(-v, sc, cen[j]);
                const float w = __builtin_amdgcn_exp2f(NEG ? fmaf(-d, d, lgx) : fmaf(d, d, lgx));
                rs[j] += w;
                rxs[j] = fmaf(w, v, rxs[j]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wsum[j] = fmaf(gyv, rs[j], wsum[j]);
            wxsum[j] = fmaf(gyv, rxs[j], wxsum[j]);
        }
    }
    float *out = y + (size_t)n * p.H * p.W;
    const int gxo = x0 + col;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int gyo = y0 + row0 + 4 * j;
        if (gyo < p.H && gxo < p.W) out[(size_t)gyo * p.W + gxo] = wxsum[j] / wsum[j];
    }
}

// ---------------------------------------------------------------------------
// Windows up to 16 taps wide: the same tile and staging, but a thread makes four adjacent
// outputs of one row and the window length is a template parameter.  A window row is then
// K + 3 consecutive staged pixels = a few aligned 16-byte LDS reads for 4 K taps (instead of
// one 4-byte read per tap), every tap index is an immediate, and the centre pixels are one
// aligned 16-byte read (staged column of output column j is j + c4 - c + a2; at a2 = c that
// is j + c4).  Lanes 0-15 of a wavefront take the 16 column groups of one row.
// ---------------------------------------------------------------------------
template <int K, bool NEG>
__global__ __launch_bounds__(256) void merit_bilateral_rows(BilatParams p, const float *__restrict__ x,
                                                           const float *__restrict__ gx,
                                                           const float *__restrict__ gy, float *__restrict__ y)
{
    constexpr int TH = 16, TW = 64;
    constexpr int C = K / 2, C4 = (C + 3) / 4 * 4, D = C4 - C;
    constexpr int NW = (D + K + 3 + 3) / 4;               // 16-byte groups of one window row
    constexpr int RH = TH + K - 1;
    extern __shared__ __align__(16) float smem[];
    float *in = smem;                                     // [RH][PI]
    float *wxl = in + RH * p.PI;                          // [K]: log2 gx
    float *wyl = wxl + K;                                 // [K]

    const int tid = threadIdx.x;
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: every XCD takes a
    // contiguous run of the raster-ordered tile list (a band of tile rows), so the halo rows and
    // the cache lines two neighbouring tiles share are fetched by one L2 once.  (With tile
    // blockIdx.x itself every neighbour sat on another XCD and the image was fetched 2.95 times.)
    const uint32_t g = xcd_band_item(blockIdx.x, (int)(gridDim.x >> 3), (int)(gridDim.x & 7));
    const uint32_t q0 = fdiv(g, p.div_tiles_x);
    const int tx = (int)(g - q0 * (uint32_t)p.tiles_x);
    const int n = (int)fdiv(q0, p.div_tiles_y);
    const int ty = (int)(q0 - (uint32_t)n * (uint32_t)p.tiles_y);
    const int x0 = tx * TW, y0 = ty * TH;
    const float *img = x + (size_t)n * p.H * p.W;

    if (tid < K) {
        wxl[tid] = __builtin_amdgcn_logf(gx[tid]);        // log2
        wyl[tid] = gy[tid];
    }
    stage_clamped(p, img, in, x0, y0, RH, tid);
    __syncthreads();

    const int q = tid & 15, row = tid >> 4;               // column group, output row
    // the scale in a vector register: a multiply-add with a scalar-register operand issues at
    // two thirds of the rate of one whose operands are all vector registers (measured)
    float sc = p.scale;
    asm("" : "+v"(sc));
    const float *base = in + row * p.PI + 4 * q;
    const float4v c4v = *reinterpret_cast<const float4v *>(base + C * p.PI + C4);
    const float cenv[4] = {c4v.x, c4v.y, c4v.z, c4v.w};
    float cen[4], wsum[4], wxsum[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) { cen[j] = cenv[j] * sc; wsum[j] = 0.0f; wxsum[j] = 0.0f; }
    float lgx[K];
#pragma unroll
    for (int a = 0; a < K; ++a) lgx[a] = wxl[a];
#pragma unroll 1
    for (int a1 = 0; a1 < K; ++a1) {
        const float gyv = wyl[a1];
        const float *rowp = base + a1 * p.PI;
        float w[4 * NW];
#pragma unroll
        for (int g = 0; g < NW; ++g) {
            const float4v h = *reinterpret_cast<const float4v *>(rowp + 4 * g);
            w[4 * g] = h.x; w[4 * g + 1] = h.y; w[4 * g + 2] = h.z; w[4 * g + 3] = h.w;
        }
        float rs[4], rxs[4];
#pragma unroll
        for (int a2 = 0; a2 < K; ++a2)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float v = w[j + D + a2];
                const float d = fmaf(-v, sc, cen[j]);
                const float e = __builtin_amdgcn_exp2f(NEG ? fmaf(-d, d, lgx[a2]) : fmaf(d, d, lgx[a2]));
                if (a2 == 0) {                            // the row sums start at the first tap
                    rs[j] = e;
                    rxs[j] = e * v;
                } else {
                    rs[j] += e;
                    rxs[j] = fmaf(e, v, rxs[j]);
                }
            }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            wsum[j] = fmaf(gyv, rs[j], wsum[j]);
            wxsum[j] = fmaf(gyv, rxs[j], wxsum[j]);
        }
    }
    const int gyo = y0 + row, gxo = x0 + 4 * q;
    if (gyo < p.H) {
        float *dst = y + (size_t)n * p.H * p.W + (size_t)gyo * p.W + gxo;
        if ((p.W & 3) == 0) {
            if (gxo < p.W)
                *reinterpret_cast<float4v *>(dst) = (float4v){wxsum[0] / wsum[0], wxsum[1] / wsum[1],
                                                               wxsum[2] / wsum[2], wxsum[3] / wsum[3]};
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (gxo + j < p.W) dst[j] = wxsum[j] / wsum[j];
        }
    }
}

template <int K>
static hipError_t launch_bil_rows(const BilatParams &p, const float *x, const float *gx, const float *gy, float *y,
                                  hipStream_t s, uint32_t grid)
{
    if (p.neg)
        hipLaunchKernelGGL((merit_bilateral_rows<K, true>), dim3(grid), dim3(256), (size_t)p.lds_bytes, s, p, x, gx, gy,
                           y);
    else
        hipLaunchKernelGGL((merit_bilateral_rows<K, false>), dim3(grid), dim3(256), (size_t)p.lds_bytes, s, p, x, gx,
                           gy, y);
    return hipGetLastError();
}

hipError_t launch_bilateral(const BilatParams &p, const float *x, const float *gx, const float *gy, float *y,
                            hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.tiles_y * p.tiles_x;
    if (grid == 0) return hipSuccess;
    const uint32_t g = (uint32_t)grid;
    switch (p.k <= 16 ? p.k : 0) {
#define MERIT_BIL_CASE(Kv) case Kv: return launch_bil_rows<Kv>(p, x, gx, gy, y, s, g)
        MERIT_BIL_CASE(1); MERIT_BIL_CASE(2); MERIT_BIL_CASE(3); MERIT_BIL_CASE(4);
        MERIT_BIL_CASE(5); MERIT_BIL_CASE(6); MERIT_BIL_CASE(7); MERIT_BIL_CASE(8);
        MERIT_BIL_CASE(9); MERIT_BIL_CASE(10); MERIT_BIL_CASE(11); MERIT_BIL_CASE(12);
        MERIT_BIL_CASE(13); MERIT_BIL_CASE(14); MERIT_BIL_CASE(15); MERIT_BIL_CASE(16);
#undef MERIT_BIL_CASE
    default: break;
    }
    if (p.neg)
        hipLaunchKernelGGL(merit_bilateral_tile<true>, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p, x,
                           gx, gy, y);
    else
        hipLaunchKernelGGL(merit_bilateral_tile<false>, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p,
                           x, gx, gy, y);
    return hipGetLastError();
}

}  // namespace merit
