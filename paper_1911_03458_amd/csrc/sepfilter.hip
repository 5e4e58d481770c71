// Separable filter for gfx950: two 1-D ranged inner products in a row (dot product, Section
// III-B Eq. 3), the window centred as in the bilateral-filter call of Section VI-A (offset -k/2):
//     t[n,p1,p2] = sum_{a2<k} kx[a2] * x[n, p1, p2 + a2 - k/2]
//     y[n,p1,p2] = sum_{a1<k} ky[a1] * t[n, p1 + a1 - k/2, p2]
// with coordinates clamped to the image.  Both passes run in one launch and the intermediate
// t never leaves LDS: 8 algorithmic bytes per pixel (one fp32 read, one fp32 written).
//
// A workgroup owns TH x 64 output pixels of one image.  The covering sub-tensor (Section IV-A,
// Eq. 9: (TH + k - 1) x (64 + k - 1), here with k rounded up to a multiple of 4 and one spare
// row / column) is staged in LDS with the clamping resolved there.  Taps go in groups of 4
// (zero taps pad the last group); a thread keeps 8 adjacent outputs in registers and slides a
// 12-element window over them, so a group costs one 16-byte LDS read (row pass) or four 4-byte
// reads (column pass) for 32 multiply-adds.  In the row pass neighbouring lanes take
// neighbouring rows; the row pitches are 4 mod 8 floats, which spreads the 16-byte accesses
// of 16 lanes over all banks (the padding layout of Section IV-B).
#include "merit_internal.h"

namespace merit {

typedef float float4v __attribute__((ext_vector_type(4)));

// G = tap groups of 4 (compile time: the sliding window then lives in renamed registers)
template <int G>
__global__ __launch_bounds__(256) void merit_sepfilter_tile(SepParams p, const float *__restrict__ x,
                                                           const float *__restrict__ kx,
                                                           const float *__restrict__ ky, float *__restrict__ y)
{
    constexpr int KPAD = 4 * G, TW = 64;
    extern __shared__ __align__(16) float smem[];
    const int RH = p.TH + KPAD;                           // staged rows (one more than any tap reaches)
    float *in = smem;                                     // [RH][PI]
    float *mid = in + RH * p.PI;                          // [RH][PM]
    float *wxl = mid + RH * p.PM;                         // [KPAD]
    float *wyl = wxl + KPAD;

    const int tid = threadIdx.x;
    const uint32_t q0 = fdiv(blockIdx.x, p.div_tiles_x);
    const int tx = (int)(blockIdx.x - q0 * (uint32_t)p.tiles_x);
    const int n = (int)fdiv(q0, p.div_tiles_y);
    const int ty = (int)(q0 - (uint32_t)n * (uint32_t)p.tiles_y);
    const int x0 = tx * TW, y0 = ty * p.TH;
    const float *img = x + (size_t)n * p.H * p.W;

    if (tid < KPAD) {
        wxl[tid] = tid < p.k ? kx[tid] : 0.0f;
        wyl[tid] = tid < p.k ? ky[tid] : 0.0f;
    }
    // staging: every element is a real (clamped) pixel, also the spare row / columns that only
    // meet zero taps, so no product is ever 0 x garbage
    for (int e = tid; e < RH * p.PI; e += 256) {
        const int r = (int)fdiv((uint32_t)e, p.div_pi);
        const int cc = e - r * p.PI;
        const int gy = min(max(y0 - p.c + r, 0), p.H - 1);
        const int gx = min(max(x0 - p.c + cc, 0), p.W - 1);
        in[e] = img[(size_t)gy * p.W + gx];
    }
    __syncthreads();

    // row pass: unit = (8-column group, staged row), rows fastest
    for (int u = tid; u < (TW / 8) * RH; u += 256) {
        const int cg = (int)fdiv((uint32_t)u, p.div_rh);
        const int r = u - cg * RH;
        const float *src = in + r * p.PI + 8 * cg;
        float win[12], acc[8];
        {
            const float4v a = *reinterpret_cast<const float4v *>(src);
            const float4v b = *reinterpret_cast<const float4v *>(src + 4);
            win[0] = a.x; win[1] = a.y; win[2] = a.z; win[3] = a.w;
            win[4] = b.x; win[5] = b.y; win[6] = b.z; win[7] = b.w;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4v h = *reinterpret_cast<const float4v *>(src + 8 + 4 * g);
            const float4v w = *reinterpret_cast<const float4v *>(wxl + 4 * g);
            win[8] = h.x; win[9] = h.y; win[10] = h.z; win[11] = h.w;
            const float wt[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] = fmaf(wt[t], win[j + t], acc[j]);
#pragma unroll
            for (int j = 0; j < 8; ++j) win[j] = win[j + 4];
        }
        float *dst = mid + r * p.PM + 8 * cg;
        float4v o0, o1;
        o0.x = acc[0]; o0.y = acc[1]; o0.z = acc[2]; o0.w = acc[3];
        o1.x = acc[4]; o1.y = acc[5]; o1.z = acc[6]; o1.w = acc[7];
        *reinterpret_cast<float4v *>(dst) = o0;
        *reinterpret_cast<float4v *>(dst + 4) = o1;
    }
    __syncthreads();

    // column pass: unit = (8-row group, column), columns fastest; stores are 256-byte row segments
    float *out = y + (size_t)n * p.H * p.W;
    for (int u = tid; u < (p.TH / 8) * TW; u += 256) {
        const int rg = u >> 6, col = u & 63;
        const float *src = mid + (8 * rg) * p.PM + col;
        float win[12], acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { win[i] = src[i * p.PM]; acc[i] = 0.0f; }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4v w = *reinterpret_cast<const float4v *>(wyl + 4 * g);
#pragma unroll
            for (int q = 0; q < 4; ++q) win[8 + q] = src[(8 + 4 * g + q) * p.PM];
            const float wt[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = fmaf(wt[t], win[i + t], acc[i]);
#pragma unroll
            for (int i = 0; i < 8; ++i) win[i] = win[i + 4];
        }
        const int gx = x0 + col;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int gy = y0 + 8 * rg + i;
            if (gy < p.H && gx < p.W) out[(size_t)gy * p.W + gx] = acc[i];
        }
    }
}

template <int G>
static hipError_t launch_sep(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                             hipStream_t s, uint32_t grid)
{
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(merit_sepfilter_tile<G>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL(merit_sepfilter_tile<G>, dim3(grid), dim3(256), (size_t)p.lds_bytes, s, p, x, kx, ky, y);
    return hipGetLastError();
}

hipError_t launch_sepfilter(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                            hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.tiles_y * p.tiles_x;
    if (grid == 0) return hipSuccess;
    const uint32_t g = (uint32_t)grid;
    switch (p.G) {
#define MERIT_SEP_CASE(Gv) case Gv: return launch_sep<Gv>(p, x, kx, ky, y, s, g)
        MERIT_SEP_CASE(1); MERIT_SEP_CASE(2); MERIT_SEP_CASE(3); MERIT_SEP_CASE(4);
        MERIT_SEP_CASE(5); MERIT_SEP_CASE(6); MERIT_SEP_CASE(7); MERIT_SEP_CASE(8);
        MERIT_SEP_CASE(9); MERIT_SEP_CASE(10); MERIT_SEP_CASE(11); MERIT_SEP_CASE(12);
        MERIT_SEP_CASE(13); MERIT_SEP_CASE(14); MERIT_SEP_CASE(15); MERIT_SEP_CASE(16);
#undef MERIT_SEP_CASE
    default: return hipErrorInvalidValue;
    }
}

}  // namespace merit
