// Depthwise convolution for gfx950: k = (n, c, oy, ox | ky, kx),
//     M(x)[p,a] = x[n, c, oy*sh + ky - ph, ox*sw + kx - pw]      (0 outside the image)
//     M(w)[p,a] = w[c, ky, kx]
// reduced with the dot product (Section III-B, Eq. 3).  The channel index is parallel, so
// there is no contraction for the matrix cores: the op moves 4 bytes per output element and
// does kh*kw multiply-adds on them — HBM-bound, plain vector arithmetic in fp32.
//
// A workgroup owns TH output rows of one (n,c) plane.  The input rows they need are one
// contiguous span of the plane (the minimal covering sub-tensor of Section IV-A, Eq. 9),
// staged in LDS with the zero padding resolved there; windows are then read branch-free.
#include "merit_internal.h"

namespace merit {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }

__device__ __forceinline__ uint16_t f2h(float f)
{
    const _Float16 h = (_Float16)f;                        // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}

// ---------------------------------------------------------------------------
// Generic kernel: any window / stride / padding / width; scalar accesses.
// LDS: [RH][pitch] halves, pitch = W + 2*pw, then the kh*kw weights as floats.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merit_dwconv_tile(DwParams p, const uint16_t *__restrict__ x,
                                                        const uint16_t *__restrict__ w, uint16_t *__restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint16_t *xl = reinterpret_cast<uint16_t *>(smem);
    float *wf = reinterpret_cast<float *>(smem + p.lds_w_offset);

    const int tid = threadIdx.x;
    const uint32_t nc = fdiv(blockIdx.x, p.div_tiles_y);
    const int strip = (int)(blockIdx.x - nc * (uint32_t)p.tiles_y);
    const int c = (int)(nc - fdiv(nc, p.div_c) * (uint32_t)p.C);
    const int oy0 = strip * p.TH;
    const int y0 = oy0 * p.sh - p.ph;
    const int rows = min(p.TH, p.OH - oy0);
    const int RH = (rows - 1) * p.sh + p.kh;
    const uint16_t *xp = x + (size_t)nc * p.H * p.W;

    for (int i = tid; i < p.kh * p.kw; i += 256) wf[i] = h2f(w[(size_t)c * p.kh * p.kw + i]);
    for (int i = tid; i < RH * p.pitch; i += 256) {
        const int r = (int)fdiv((uint32_t)i, p.div_pitch);
        const int col = i - r * p.pitch;
        const int gy = y0 + r, gx = col - p.pw;
        uint16_t v = 0;
        if (gy >= 0 && gy < p.H && gx >= 0 && gx < p.W) v = xp[(size_t)gy * p.W + gx];
        xl[i] = v;
    }
    __syncthreads();

    uint16_t *yp = y + (size_t)nc * p.OH * p.OW;
    for (int o = tid; o < rows * p.OW; o += 256) {
        const int ty = (int)fdiv((uint32_t)o, p.div_ow);
        const int ox = o - ty * p.OW;
        const uint16_t *win = xl + (ty * p.sh) * p.pitch + ox * p.sw;
        float acc = 0.0f;
        for (int ky = 0; ky < p.kh; ++ky)
            for (int kx = 0; kx < p.kw; ++kx) acc = fmaf(h2f(win[ky * p.pitch + kx]), wf[ky * p.kw + kx], acc);
        yp[(size_t)(oy0 + ty) * p.OW + ox] = f2h(acc);
    }
}

// ---------------------------------------------------------------------------
// 3x3, stride 1, padding 1, W % 8 == 0 (the MobileNet layer).  LDS rows are
// [8 zero halves][W halves][8 zero halves], so every 16-byte chunk is aligned; rows are
// copied with 16-byte loads.  A thread makes 8 adjacent outputs from three aligned 16-byte
// reads per window row (it needs the last half of the chunk on its left, its own chunk and
// the first half of the chunk on its right) and stores them as one 16-byte run.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merit_dwconv_rows_k3s1p1(DwParams p, const uint16_t *__restrict__ x,
                                                               const uint16_t *__restrict__ w,
                                                               uint16_t *__restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *xl = reinterpret_cast<uint4 *>(smem);            // [RH][pitch8] chunks of 8 halves
    const int tid = threadIdx.x;
    const uint32_t nc = fdiv(blockIdx.x, p.div_tiles_y);
    const int strip = (int)(blockIdx.x - nc * (uint32_t)p.tiles_y);
    const int c = (int)(nc - fdiv(nc, p.div_c) * (uint32_t)p.C);
    const int oy0 = strip * p.TH;
    const int rows = min(p.TH, p.OH - oy0);
    const int RH = rows + 2;
    const int W8 = p.W >> 3, pitch8 = W8 + 2;
    const uint16_t *xp = x + (size_t)nc * p.H * p.W;

    // weights: nine wave-uniform loads
    float wk[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) wk[i] = h2f(w[(size_t)c * 9 + i]);

    // batches of SB chunks per thread, every load issued before the first LDS write (one memory
    // round trip per batch); a chunk outside the plane re-reads the plane's first bytes and is zeroed
    constexpr int SB = 4;
    const int total = RH * pitch8;
    for (int i0 = tid; i0 < total; i0 += 256 * SB) {
        uint4 v[SB];
        bool in[SB];
#pragma unroll
        for (int b = 0; b < SB; ++b) {
            const int i = min(i0 + 256 * b, total - 1);
            const int r = (int)fdiv((uint32_t)i, p.div_pitch);
            const int c8 = i - r * pitch8;                  // 0 and W8+1 are the zero chunks
            const int gy = oy0 - 1 + r;
            in[b] = gy >= 0 && gy < p.H && c8 >= 1 && c8 <= W8;
            v[b] = *reinterpret_cast<const uint4 *>(in[b] ? xp + (size_t)gy * p.W + 8 * (c8 - 1) : xp);
        }
#pragma unroll
        for (int b = 0; b < SB; ++b)
            if (i0 + 256 * b < total) xl[i0 + 256 * b] = in[b] ? v[b] : make_uint4(0, 0, 0, 0);
    }
    __syncthreads();

    uint16_t *yp = y + (size_t)nc * p.OH * p.OW;
    for (int o = tid; o < rows * W8; o += 256) {
        const int ty = (int)fdiv((uint32_t)o, p.div_ow);     // div_ow holds W8 for this variant
        const int x8 = o - ty * W8;
        float acc[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = 0.0f;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const uint4 *row = xl + (ty + ky) * pitch8 + x8;  // chunks x8 (left), x8+1 (own), x8+2 (right)
            const half8 l = __builtin_bit_cast(half8, row[0]);
            const half8 m = __builtin_bit_cast(half8, row[1]);
            const half8 r = __builtin_bit_cast(half8, row[2]);
            float v[10];
            v[0] = (float)l[7];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[1 + k] = (float)m[k];
            v[9] = (float)r[0];
#pragma unroll
            for (int k = 0; k < 8; ++k)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) acc[k] = fmaf(v[k + kx], wk[ky * 3 + kx], acc[k]);
        }
        uint4 out;
        out.x = (uint32_t)f2h(acc[0]) | ((uint32_t)f2h(acc[1]) << 16);
        out.y = (uint32_t)f2h(acc[2]) | ((uint32_t)f2h(acc[3]) << 16);
        out.z = (uint32_t)f2h(acc[4]) | ((uint32_t)f2h(acc[5]) << 16);
        out.w = (uint32_t)f2h(acc[6]) | ((uint32_t)f2h(acc[7]) << 16);
        *reinterpret_cast<uint4 *>(yp + (size_t)(oy0 + ty) * p.OW + 8 * x8) = out;
    }
}

hipError_t launch_dwconv(const DwParams &p, const void *x, const void *w, void *y, hipStream_t s)
{
    const int64_t grid = (int64_t)p.NC * p.tiles_y;
    if (grid == 0) return hipSuccess;
    const uint16_t *xs = reinterpret_cast<const uint16_t *>(x);
    const uint16_t *ws = reinterpret_cast<const uint16_t *>(w);
    uint16_t *ys = reinterpret_cast<uint16_t *>(y);
    if (p.lds_bytes > 64 * 1024) {     // wide rows: more dynamic LDS than a kernel gets by default
        static std::atomic<int> raised_rows{0}, raised_tile{0};
        const bool rows = p.variant == DW_ROWS_K3S1P1;
        if (hipError_t e = raise_lds_limit_once(rows ? reinterpret_cast<const void *>(merit_dwconv_rows_k3s1p1)
                                                     : reinterpret_cast<const void *>(merit_dwconv_tile),
                                                rows ? raised_rows : raised_tile);
            e != hipSuccess)
            return e;
    }
    if (p.variant == DW_ROWS_K3S1P1)
        hipLaunchKernelGGL(merit_dwconv_rows_k3s1p1, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p, xs, ws, ys);
    else
        hipLaunchKernelGGL(merit_dwconv_tile, dim3((uint32_t)grid), dim3(256), (size_t)p.lds_bytes, s, p, xs, ws, ys);
    return hipGetLastError();
}

const char *dwconv_kernel_name(const DwParams &p)
{
    return p.variant == DW_ROWS_K3S1P1 ? "merit_dwconv_rows_k3s1p1" : "merit_dwconv_tile";
}

}  // namespace merit
