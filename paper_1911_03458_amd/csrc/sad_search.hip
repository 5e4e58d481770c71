// Block-matching motion estimation for gfx950: two-level ranged inner product.
//
// k = (by, bx | dy, dx, i, j).  Inner level: L1 distance (Section III-B, Eq. 4)
// between the current block and the reference block displaced by the search
// indices (index pattern of Section III-C, Eq. 8):
//     M(cur)[p,a] = cur[by*B + i,          bx*B + j         ]
//     M(ref)[p,a] = ref[by*B + i + dy - R, bx*B + j + dx - R]   (clamped to the frame)
// Outer level: min / argmin over (dy,dx), ties to the lowest raster index.
//
// The reference search window (B+2R)^2, i.e. the minimal covering sub-tensor of
// Section IV-A, Eq. 9, is staged once in LDS with the clamping resolved there;
// candidates then read it branch-free.  Four pixels per lane-op with v_sad_u8.
// The (sad, raster index) pair is packed into one u32 key so that integer min
// gives the lexicographic minimum, reduced across the wavefront with DPP.
#include "merit_internal.h"

namespace merit {

constexpr int KEY_SHIFT = 14;                 // raster index < 2^14 (R <= 63)
constexpr uint32_t KEY_MASK = (1u << KEY_SHIFT) - 1u;

// min over the 64 lanes of a wavefront; the result is valid in lane 63.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ uint32_t dpp_min_step(uint32_t v)
{
    // lanes whose source is disabled or out of range keep the identity 0xffffffff
    const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)0xffffffff, (int)v, CTRL, ROW_MASK, 0xf, false);
    return o < v ? o : v;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v)
{
    v = dpp_min_step<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
    v = dpp_min_step<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
    v = dpp_min_step<0x141, 0xf>(v);   // row_half_mirror
    v = dpp_min_step<0x140, 0xf>(v);   // row_mirror: every lane holds its row's min
    v = dpp_min_step<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_min_step<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Stage the clamped search window of block (by,bx) as bytes win[wy*pitch + wx],
// wy,wx in [0, B+2R), four bytes per thread-iteration.
__device__ __forceinline__ void stage_window(const SadParams &p, const uint8_t *__restrict__ ref,
                                             uint32_t *win32, int gy0, int gx0, int rows, int cols4,
                                             FastDiv div_cols4, int pitch4, int tid, int nthreads)
{
    const bool aligned = ((gx0 & 3) == 0) && ((p.W & 3) == 0);
    const int n = rows * cols4;
    for (int i = tid; i < n; i += nthreads) {
        const int wy = (int)fdiv((uint32_t)i, div_cols4);
        const int w4 = i - wy * cols4;
        const int gy = min(max(gy0 + wy, 0), p.H - 1);
        const int gx = gx0 + 4 * w4;
        const uint8_t *row = ref + (size_t)gy * p.W;
        uint32_t v;
        if (aligned && gx >= 0 && gx + 3 < p.W) {
            v = *reinterpret_cast<const uint32_t *>(row + gx);
        } else {
            v = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int cx = min(max(gx + b, 0), p.W - 1);
                v |= (uint32_t)row[cx] << (8 * b);
            }
        }
        win32[wy * pitch4 + w4] = v;
    }
}

// ---------------------------------------------------------------------------
// Generic kernel: one workgroup per block, one lane per candidate (strided).
// Any B that is a multiple of 4 (<= 32) and any R <= 63.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void merit_sad_generic(SadParams p, const uint8_t *__restrict__ cur,
                                                        const uint8_t *__restrict__ ref,
                                                        int32_t *__restrict__ sad, int32_t *__restrict__ mv)
{
    extern __shared__ __align__(16) uint32_t lds32[];
    const int tid = threadIdx.x;
    const int pitch4 = p.pitch >> 2;
    const int B4 = p.B >> 2;
    uint32_t *win32 = lds32;                                  // [win][pitch4] (+1 dword slack)
    uint32_t *cur32 = lds32 + p.win * pitch4 + 1;             // [B][B4]
    uint32_t *red = cur32 + p.B * B4;                         // [4]

    const uint32_t blk = blockIdx.x;
    const int by = (int)(blk / (uint32_t)p.nbx);
    const int bx = (int)(blk - (uint32_t)by * p.nbx);

    stage_window(p, ref, win32, by * p.B - p.R, bx * p.B - p.R, p.win, (p.win + 3) >> 2,
                 p.div_win4, pitch4, tid, 256);
    for (int i = tid; i < p.B * B4; i += 256) {
        const int r = i / B4, c4 = i - r * B4;
        cur32[i] = *reinterpret_cast<const uint32_t *>(cur + (size_t)(by * p.B + r) * p.W + bx * p.B + 4 * c4);
    }
    __syncthreads();

    uint32_t best = 0xffffffffu;
    const int ncand = p.n * p.n;
    for (int c = tid; c < ncand; c += 256) {
        const int dyi = (int)fdiv((uint32_t)c, p.div_n);       // dy + R
        const int dxi = c - dyi * p.n;                         // dx + R
        uint32_t acc = 0;
        for (int i = 0; i < p.B; ++i) {
            const int byte0 = (dyi + i) * p.pitch + dxi;
            const uint32_t sh = (uint32_t)(byte0 & 3);
            const uint32_t *w = win32 + (byte0 >> 2);
            uint32_t lo = w[0];
            for (int j4 = 0; j4 < B4; ++j4) {
                const uint32_t hi = w[j4 + 1];
                const uint32_t r4 = __builtin_amdgcn_alignbyte(hi, lo, sh);
                acc = __builtin_amdgcn_sad_u8(cur32[i * B4 + j4], r4, acc);
                lo = hi;
            }
        }
        const uint32_t key = (acc << KEY_SHIFT) | (uint32_t)c;
        best = key < best ? key : best;
    }
    best = wave_min_u32(best);
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) {
        uint32_t k = red[0];
        for (int w = 1; w < 4; ++w) k = red[w] < k ? red[w] : k;
        const uint32_t c = k & KEY_MASK;
        const int dyi = (int)(c / (uint32_t)p.n);
        sad[blk] = (int32_t)(k >> KEY_SHIFT);
        mv[2 * blk + 0] = dyi - p.R;
        mv[2 * blk + 1] = (int)c - dyi * p.n - p.R;
    }
}

// ---------------------------------------------------------------------------
hipError_t launch_sad(const SadParams &p, const uint8_t *cur, const uint8_t *ref, int32_t *sad,
                      int32_t *mv, hipStream_t s)
{
    const uint32_t nblocks = (uint32_t)(p.nby * p.nbx);
    if (nblocks == 0) return hipSuccess;
    const int pitch4 = p.pitch >> 2;
    const size_t lds_bytes = (size_t)(p.win * pitch4 + 1 + p.B * (p.B >> 2) + 4) * 4;
    hipLaunchKernelGGL(merit_sad_generic, dim3(nblocks), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
    return hipGetLastError();
}

const char *sad_kernel_name(const SadParams &p)
{
    (void)p;
    return "merit_sad_generic";
}

}  // namespace merit
