// Separable filter for gfx950: two 1-D ranged inner products in a row (dot product, Section
// III-B Eq. 3), the window centred as in the bilateral-filter call of Section VI-A (offset -k/2):
//     t[n,p1,p2] = sum_{a2<k} kx[a2] * x[n, p1, p2 + a2 - k/2]
//     y[n,p1,p2] = sum_{a1<k} ky[a1] * t[n, p1 + a1 - k/2, p2]
// with coordinates clamped to the image.  Both passes run in one launch and the intermediate
// t never leaves LDS: 8 algorithmic bytes per pixel (one fp32 read, one fp32 written).
//
// A workgroup owns TH x 64 output pixels of one image.  The covering sub-tensor (Section IV-A,
// Eq. 9: (TH + k - 1) x (64 + k - 1)) is staged in LDS with the clamping resolved there.  A
// row-pass thread keeps 8 adjacent outputs of one staged row in registers and reads the
// 8 + k - 1 inputs they need as 16-byte runs; a column-pass thread keeps a 4 x 4 patch and
// reads k + 3 runs of four columns: 8k and 16k multiply-adds for that many 16-byte reads.
// In the row pass neighbouring lanes take neighbouring rows; the row pitches are 4 mod 8
// floats, which spreads the 16-byte accesses of 16 lanes over all banks (the padding layout
// of Section IV-B).
//
// The staged columns start at x0 - c4, c4 = k/2 rounded up to 4, so that (for W % 4 == 0) every
// group of four staged columns is one aligned 16-byte run of the image, entirely inside it or
// entirely outside (then it is four copies of the edge pixel): the staging is 16-byte loads
// without a branch, and the row pass reads its window c4 - k/2 columns further right.
#include "merit_internal.h"

namespace merit {

typedef float float4v __attribute__((ext_vector_type(4)));

// K = window length (compile time: every tap index is an immediate, the sliding windows live
// in renamed registers and no zero tap is multiplied)
template <int K>
__global__ __launch_bounds__(256) void merit_sepfilter_tile(SepParams p, const float *__restrict__ x,
                                                           const float *__restrict__ kx,
                                                           const float *__restrict__ ky, float *__restrict__ y)
{
    constexpr int TW = 64;
    constexpr int C = K / 2, C4 = (C + 3) / 4 * 4, D = C4 - C;    // staged column 0 = image column x0 - C4
    constexpr int NWR = (D + 8 + K - 1 + 3) / 4;                  // 16-byte groups a row-pass unit reads
    constexpr int K4 = (K + 3) / 4;
    extern __shared__ __align__(16) float smem[];
    const int RH = p.TH + K - 1;                          // staged rows
    float *in = smem;                                     // [RH][PI]
    float *mid = in + RH * p.PI;                          // [RH][PM]
    float *wxl = mid + RH * p.PM;                         // [4*K4]
    float *wyl = wxl + 4 * K4;                            // [4*K4]

    const int tid = threadIdx.x;
    const uint32_t q0 = fdiv(blockIdx.x, p.div_tiles_x);
    const int tx = (int)(blockIdx.x - q0 * (uint32_t)p.tiles_x);
    const int n = (int)fdiv(q0, p.div_tiles_y);
    const int ty = (int)(q0 - (uint32_t)n * (uint32_t)p.tiles_y);
    const int x0 = tx * TW, y0 = ty * p.TH;
    const float *img = x + (size_t)n * p.H * p.W;

    if (tid < 4 * K4) {
        wxl[tid] = tid < K ? kx[min(tid, K - 1)] : 0.0f;
        wyl[tid] = tid < K ? ky[min(tid, K - 1)] : 0.0f;
    }
    // staging: every element is a real (clamped) pixel.  A thread owns one 4-column group of
    // the staged rows r = tid / LPR + (256 / LPR) j; SB rows per batch, every load of a batch
    // issued before the first LDS write (one memory round trip per batch).
    constexpr int SB = 8;
    const int P4 = p.PI >> 2;
    if ((p.W & 3) == 0) {
        const int W4 = p.W >> 2;
        const int lg = P4 <= 32 ? 5 : 6;                  // lanes per staged row: 32 or 64
        const int cg = tid & ((1 << lg) - 1);
        const int g4 = ((x0 - C4) >> 2) + cg;             // image 4-column group (may be outside)
        const bool live = cg < P4;
        const bool inside = g4 >= 0 && g4 < W4;
        const bool left = g4 < 0;
        const float *col = img + 4 * min(max(g4, 0), W4 - 1);
        const int rstep = 256 >> lg;
        for (int r0 = tid >> lg; r0 < RH; r0 += rstep * SB) {
            float4v v[SB];
#pragma unroll
            for (int b = 0; b < SB; ++b) {
                const int gy = min(max(y0 - C + r0 + rstep * b, 0), p.H - 1);
                v[b] = *reinterpret_cast<const float4v *>(col + (size_t)gy * p.W);
            }
#pragma unroll
            for (int b = 0; b < SB; ++b) {
                const int r = r0 + rstep * b;
                const float edge = left ? v[b].x : v[b].w;
                float4v o;
                o.x = inside ? v[b].x : edge; o.y = inside ? v[b].y : edge;
                o.z = inside ? v[b].z : edge; o.w = inside ? v[b].w : edge;
                if (live && r < RH) reinterpret_cast<float4v *>(in)[r * P4 + cg] = o;
            }
        }
    } else {
        const int total = RH * p.PI;
        for (int e = tid; e < total; e += 256) {
            const int r = e / p.PI;
            const int cc = e - r * p.PI;
            const int gy = min(max(y0 - C + r, 0), p.H - 1);
            const int gx = min(max(x0 - C4 + cc, 0), p.W - 1);
            in[e] = img[(size_t)gy * p.W + gx];
        }
    }
    __syncthreads();

    // row pass: unit = (8-column group, staged row), rows fastest; output column j of the unit
    // = sum_a kx[a] * staged column (8 cg + j + D + a)
    for (int u = tid; u < (TW / 8) * RH; u += 256) {
        const int cg = (int)fdiv((uint32_t)u, p.div_rh);
        const int r = u - cg * RH;
        const float *src = in + r * p.PI + 8 * cg;
        float win[4 * NWR], acc[8];
#pragma unroll
        for (int g = 0; g < NWR; ++g) {
            const float4v h = *reinterpret_cast<const float4v *>(src + 4 * g);
            win[4 * g] = h.x; win[4 * g + 1] = h.y; win[4 * g + 2] = h.z; win[4 * g + 3] = h.w;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int g = 0; g < K4; ++g) {
            const float4v w = *reinterpret_cast<const float4v *>(wxl + 4 * g);
            const float wt[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int t = 0; t < 4; ++t)
                if (4 * g + t < K) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc[j] = fmaf(wt[t], win[j + D + 4 * g + t], acc[j]);
                }
        }
        float *dst = mid + r * p.PM + 8 * cg;
        float4v o0, o1;
        o0.x = acc[0]; o0.y = acc[1]; o0.z = acc[2]; o0.w = acc[3];
        o1.x = acc[4]; o1.y = acc[5]; o1.z = acc[6]; o1.w = acc[7];
        *reinterpret_cast<float4v *>(dst) = o0;
        *reinterpret_cast<float4v *>(dst + 4) = o1;
    }
    __syncthreads();

    // column pass: unit = 4 rows x 4 columns, column groups fastest: 16-byte LDS reads and
    // 16-byte stores.  Row q of the K + 3 rows a unit reads feeds output row i with tap q - i.
    float *out = y + (size_t)n * p.H * p.W;
    const bool vec_out = (p.W & 3) == 0;
    for (int u = tid; u < (p.TH / 4) * (TW / 4); u += 256) {
        const int rg = u >> 4, c4 = u & 15;
        const float *src = mid + (4 * rg) * p.PM + 4 * c4;
        float4v acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = (float4v){0.0f, 0.0f, 0.0f, 0.0f};
        float wt[4 * K4];
#pragma unroll
        for (int g = 0; g < K4; ++g) {
            const float4v w = *reinterpret_cast<const float4v *>(wyl + 4 * g);
            wt[4 * g] = w.x; wt[4 * g + 1] = w.y; wt[4 * g + 2] = w.z; wt[4 * g + 3] = w.w;
        }
#pragma unroll
        for (int q = 0; q < K + 3; ++q) {
            const float4v v = *reinterpret_cast<const float4v *>(src + q * p.PM);
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (q - i >= 0 && q - i < K) {
                    acc[i].x = fmaf(wt[q - i], v.x, acc[i].x);
                    acc[i].y = fmaf(wt[q - i], v.y, acc[i].y);
                    acc[i].z = fmaf(wt[q - i], v.z, acc[i].z);
                    acc[i].w = fmaf(wt[q - i], v.w, acc[i].w);
                }
        }
        const int gx = x0 + 4 * c4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int gy = y0 + 4 * rg + i;
            if (gy >= p.H) continue;
            float *dst = out + (size_t)gy * p.W + gx;
            if (vec_out) {
                if (gx < p.W) *reinterpret_cast<float4v *>(dst) = acc[i];
            } else {
                if (gx < p.W) dst[0] = acc[i].x;
                if (gx + 1 < p.W) dst[1] = acc[i].y;
                if (gx + 2 < p.W) dst[2] = acc[i].z;
                if (gx + 3 < p.W) dst[3] = acc[i].w;
            }
        }
    }
}

template <int K>
static hipError_t launch_sep(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                             hipStream_t s, uint32_t grid)
{
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(merit_sepfilter_tile<K>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL(merit_sepfilter_tile<K>, dim3(grid), dim3(256), (size_t)p.lds_bytes, s, p, x, kx, ky, y);
    return hipGetLastError();
}

hipError_t launch_sepfilter(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                            hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.tiles_y * p.tiles_x;
    if (grid == 0) return hipSuccess;
    const uint32_t g = (uint32_t)grid;
    switch (p.k) {
#define MERIT_SEP_CASE(Kv) case Kv: return launch_sep<Kv>(p, x, kx, ky, y, s, g)
#define MERIT_SEP_CASE8(B)                                                                           \
    MERIT_SEP_CASE(B + 1); MERIT_SEP_CASE(B + 2); MERIT_SEP_CASE(B + 3); MERIT_SEP_CASE(B + 4);      \
    MERIT_SEP_CASE(B + 5); MERIT_SEP_CASE(B + 6); MERIT_SEP_CASE(B + 7); MERIT_SEP_CASE(B + 8)
        MERIT_SEP_CASE8(0); MERIT_SEP_CASE8(8); MERIT_SEP_CASE8(16); MERIT_SEP_CASE8(24);
#undef MERIT_SEP_CASE8
#undef MERIT_SEP_CASE
    default: return hipErrorInvalidValue;
    }
}

}  // namespace merit
