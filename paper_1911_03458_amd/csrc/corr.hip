// Correlation layer for gfx950 (Section III-C, Eq. 8):
//     M(I1)[p,a] = I1[b, a1, p1, p2]
//     M(I2)[p,a] = I2[b, a1, p1 + (p3-R)*sd, p2 + (p4-R)*sd]      (0 outside the image)
// with k = (b, p1, p2, p3, p4 | a1) and the dot product over the channel index a1
// (Section III-B, Eq. 3).  Output y[b,p1,p2,p3,p4], binary16, fp32 accumulation.
//
// A workgroup owns (b, p1, p3, a run of 64 pixels p2): one row of the first tensor and one
// (displaced) row of the second.  Both are staged in LDS with the channel axis innermost,
// eight channels = 16 bytes per pixel, transposed in registers on the way (v_perm_b32), so
// that a lane reads eight channels of a pixel with one LDS load and reduces them with four
// v_dot2 (two fp16 products accumulated in fp32 each).  Lane = pixel p2; the four wavefronts
// split the column displacements p4; a lane keeps one accumulator per p4 it owns.  Channels
// go through LDS in passes of `chg` groups of eight.  Needs W % 8 == 0 and R <= 15.
#include "merit_internal.h"

namespace merit {

typedef _Float16 half2c __attribute__((ext_vector_type(2)));

// Stage, for channel groups [chi0, chi0+ng), 8-pixel units of both rows of one pass:
//   first tensor,  row p1, columns px0 + 8*x8 (x8 < npx8)          -> a1l[g*64 + col]
//   second tensor, row yy, columns gx2 + 8*x8 (x8 < cols2/8)       -> a2l[g*cols2 + col]
// each as 8 channels of one pixel per 16 bytes (transposed in registers).  All units of a pass
// are one list, XB per thread, and every global load of a batch is issued before the first
// use, so that a pass costs one memory round trip (at most two for large passes).  8-column
// units outside the row (starts are multiples of 8, W % 8 == 0) and missing channels give zeros.
// Column swizzle of the staged rows (the XOR layout of Section IV-B): inside every run of 8
// columns the position is XORed with the run's index.  A staging thread writes the 8 pixels
// of one run, its neighbours the adjacent runs, 128 bytes apart: unswizzled, eight lanes
// would hit two bank groups; swizzled they hit eight.  Readers of consecutive columns still
// see (almost always) distinct bank groups.
__device__ __forceinline__ int swz(int col) { return col ^ ((col >> 3) & 7); }

__device__ __forceinline__ void stage_pass_8ch(const CorrParams &p, const uint16_t *__restrict__ x1,
                                               const uint16_t *__restrict__ x2, uint4 *a1l, uint4 *a2l, int b,
                                               int p1, int yy, int px0, int npx8, int gx2, int chi0, int ng,
                                               int tid)
{
    const int u2 = p.cols2 >> 3;                 // units per group of the second tensor
    const int per_g = npx8 + u2;
    const int nu = ng * per_g;
    const size_t chstride = (size_t)p.H * p.W;
    constexpr int XB = 3;
    for (int u0 = tid; u0 < nu; u0 += 256 * XB) {
        uint32_t v[XB][8][4];
#pragma unroll
        for (int k = 0; k < XB; ++k) {
            const int u = min(u0 + 256 * k, nu - 1);
            const int g = u / per_g;
            const int r = u - g * per_g;
            const bool second = r >= npx8;
            const int gx = second ? gx2 + 8 * (r - npx8) : px0 + 8 * r;
            const int gy = second ? yy : p1;
            const bool colok = gx >= 0 && gx < p.W;
            const int c0 = (chi0 + g) * 8;
            const uint16_t *xs = second ? x2 : x1;
            const uint16_t *src = xs + (((size_t)b * p.C + c0) * p.H + gy) * p.W + (colok ? gx : 0);
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const bool ok = colok && (c0 + c < p.C);
                // branch-free: a missing element re-reads the tensor's first bytes and is zeroed
                const uint4 t4 = *reinterpret_cast<const uint4 *>(ok ? src + c * chstride : xs);
                v[k][c][0] = ok ? t4.x : 0u; v[k][c][1] = ok ? t4.y : 0u;
                v[k][c][2] = ok ? t4.z : 0u; v[k][c][3] = ok ? t4.w : 0u;
            }
        }
#pragma unroll
        for (int k = 0; k < XB; ++k) {
            const int u = u0 + 256 * k;
            if (u >= nu) break;
            const int g = u / per_g;
            const int r = u - g * per_g;
            const int run = (r >= npx8) ? r - npx8 : r;
            uint4 *d4 = (r >= npx8) ? a2l + g * p.cols2 + 8 * run : a1l + g * 64 + 8 * run;
#pragma unroll
            for (int px = 0; px < 8; ++px) {
                const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
                uint32_t d[4];
#pragma unroll
                for (int qq = 0; qq < 4; ++qq)
                    d[qq] = __builtin_amdgcn_perm(v[k][2 * qq + 1][px >> 1], v[k][2 * qq][px >> 1], sel);
                d4[px ^ (run & 7)] = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
    }
}

__device__ __forceinline__ float dot8(const uint4 &a, const uint4 &b, float acc)
{
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2c, a.x), __builtin_bit_cast(half2c, b.x), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2c, a.y), __builtin_bit_cast(half2c, b.y), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2c, a.z), __builtin_bit_cast(half2c, b.z), acc, false);
    acc = __builtin_amdgcn_fdot2(__builtin_bit_cast(half2c, a.w), __builtin_bit_cast(half2c, b.w), acc, false);
    return acc;
}

// NACC = column displacements per wavefront = ceil((2R+1) / 4).
template <int NACC>
__global__ __launch_bounds__(256) void merit_corr_dot(CorrParams p, const uint16_t *__restrict__ x1,
                                                      const uint16_t *__restrict__ x2, uint16_t *__restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *a1l = reinterpret_cast<uint4 *>(smem);                 // [chg][64]
    uint4 *a2l = a1l + p.chg * 64;                                // [chg][cols2]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // Consecutive hardware workgroup ids go to the 8 XCDs in turn, each with an L2 of its own.
    // XCD x takes the x-th contiguous eighth of the work list, i.e. a band of image rows: its
    // L2 then fetches that band and its halo rows of the second tensor, not both whole tensors.
    const uint32_t xcd = blockIdx.x & 7u, slot = blockIdx.x >> 3;
    uint32_t g = xcd * (uint32_t)p.xq + min(xcd, (uint32_t)p.xr) + slot;
    // work item -> (b, p1, p3, pixel chunk), chunk fastest
    const uint32_t q0 = fdiv(g, p.div_xchunks);
    const int xc = (int)(g - q0 * (uint32_t)p.xchunks);
    const uint32_t q1 = fdiv(q0, p.div_n);
    const int p3 = (int)(q0 - q1 * (uint32_t)p.n);
    const int b = (int)fdiv(q1, p.div_h);
    const int p1 = (int)(q1 - (uint32_t)b * (uint32_t)p.H);

    const int px0 = xc * 64;
    const int p2 = px0 + lane;
    const int yy = p1 + (p3 - p.R) * p.sd;
    const bool rowok = yy >= 0 && yy < p.H;
    const int npx8 = min(8, (p.W - px0) >> 3);                    // 8-pixel units of the first tensor's chunk
    const int gx2 = px0 - p.lead;                                 // first staged column of the second tensor

    // this lane's columns in the staged second row, one per displacement it owns:
    // p2 + (p4-R)*sd - gx2 with p4 = wave + 4j (past the last displacement: the last one again,
    // computed twice and stored once); lanes past the row end read column 0 of their own
    int col[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j)
        col[j] = swz(min(lane, p.W - 1 - px0) + p.lead + (min(wave + 4 * j, p.n - 1) - p.R) * p.sd);

    const int col1 = swz(min(lane, p.W - 1 - px0));

    float acc[NACC];
#pragma unroll
    for (int j = 0; j < NACC; ++j) acc[j] = 0.0f;

    if (rowok) {                                                  // uniform: else every product is 0
        for (int chi0 = 0; chi0 < p.nchi; chi0 += p.chg) {
            const int ng = min(p.chg, p.nchi - chi0);
            __syncthreads();                                      // previous pass has been read
            stage_pass_8ch(p, x1, x2, a1l, a2l, b, p1, yy, px0, npx8, gx2, chi0, ng, tid);
            __syncthreads();
            // no branch inside: all reads of two channel groups are issued before their use
            int gi = 0;
            for (; gi + 2 <= ng; gi += 2) {
                uint4 a[2], bq[2][NACC];
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    a[e] = a1l[(gi + e) * 64 + col1];
#pragma unroll
                    for (int j = 0; j < NACC; ++j) bq[e][j] = a2l[(gi + e) * p.cols2 + col[j]];
                }
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int j = 0; j < NACC; ++j) acc[j] = dot8(a[e], bq[e][j], acc[j]);
            }
            if (gi < ng) {
                const uint4 a = a1l[gi * 64 + col1];
#pragma unroll
                for (int j = 0; j < NACC; ++j) acc[j] = dot8(a, a2l[gi * p.cols2 + col[j]], acc[j]);
            }
        }
    }
    if (p2 < p.W) {
        uint16_t *yo = y + ((((size_t)b * p.H + p1) * p.W + p2) * p.n + p3) * p.n;
#pragma unroll
        for (int j = 0; j < NACC; ++j) {
            const int p4 = wave + 4 * j;
            if (p4 < p.n) {
                const _Float16 h = (_Float16)acc[j];              // round to nearest even
                yo[p4] = __builtin_bit_cast(uint16_t, h);
            }
        }
    }
}

size_t corr_lds_bytes(const CorrParams &p)
{
    return (size_t)p.chg * (64 + p.cols2) * 16;
}

template <int NACC>
static hipError_t launch_corr(const CorrParams &p, const void *x1, const void *x2, void *y, hipStream_t s,
                              uint32_t grid)
{
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(merit_corr_dot<NACC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL(merit_corr_dot<NACC>, dim3(grid), dim3(256), corr_lds_bytes(p), s, p,
                       reinterpret_cast<const uint16_t *>(x1), reinterpret_cast<const uint16_t *>(x2),
                       reinterpret_cast<uint16_t *>(y));
    return hipGetLastError();
}

hipError_t launch_correlation(const CorrParams &p, const void *x1, const void *x2, void *y, hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.H * p.n * p.xchunks;
    if (grid == 0) return hipSuccess;
    const uint32_t gx = (uint32_t)grid;
    switch ((p.n + 3) / 4) {
    case 1: return launch_corr<1>(p, x1, x2, y, s, gx);
    case 2: return launch_corr<2>(p, x1, x2, y, s, gx);
    case 3: return launch_corr<3>(p, x1, x2, y, s, gx);
    case 4: return launch_corr<4>(p, x1, x2, y, s, gx);
    case 5: return launch_corr<5>(p, x1, x2, y, s, gx);
    case 6: return launch_corr<6>(p, x1, x2, y, s, gx);
    case 7: return launch_corr<7>(p, x1, x2, y, s, gx);
    case 8: return launch_corr<8>(p, x1, x2, y, s, gx);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace merit
