// Bilateral filter for gfx950: the strategy class and call of Section VI-A (Listings 2, 3) on a
// k x k window centred with offset -k/2 on both window indices,
//     PreLoop : wsum = wxsum = 0; center = x[n,p1,p2]
//     Loop    : v = x[n, p1 + a1 - k/2, p2 + a2 - k/2];  d = center - v
//               w = exp(d*d*norm) * gy[a1] * gx[a2];  wsum += w;  wxsum += w*v
//     PostLoop: y[n,p1,p2] = wxsum / wsum
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
    const uint32_t q0 = fdiv(blockIdx.x, p.div_tiles_x);
    const int tx = (int)(blockIdx.x - q0 * (uint32_t)p.tiles_x);
    const int n = (int)fdiv(q0, p.div_tiles_y);
    const int ty = (int)(q0 - (uint32_t)n * (uint32_t)p.tiles_y);
    const int x0 = tx * TW, y0 = ty * TH;
    const float *img = x + (size_t)n * p.H * p.W;

    if (tid < p.k) {
        wxl[tid] = __builtin_amdgcn_logf(gx[tid]);        // log2
        wyl[tid] = gy[tid];
    }
    // staging: every element is a real (clamped) pixel
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

hipError_t launch_bilateral(const BilatParams &p, const float *x, const float *gx, const float *gy, float *y,
                            hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.tiles_y * p.tiles_x;
    if (grid == 0) return hipSuccess;
    if (p.neg)
        hipLaunchKernelGGL(merit_bilateral_tile<true>, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p, x,
                           gx, gy, y);
    else
        hipLaunchKernelGGL(merit_bilateral_tile<false>, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p,
                           x, gx, gy, y);
    return hipGetLastError();
}

}  // namespace merit
