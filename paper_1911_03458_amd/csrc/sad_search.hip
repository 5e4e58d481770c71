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

// v + (the lanes below in the same group of G = 8 or 16 lanes): the last lane of every
// group holds the group's sum.  Lanes shifted in from outside a 16-lane row read 0.
template <int G>
__device__ __forceinline__ uint32_t group_sum_u32(uint32_t v)
{
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
    if (G == 16) v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
    return v;
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

    const uint32_t blk = xcd_band_item(blockIdx.x, p.xq, p.xr);   // a band of block rows per XCD
    const int by = (int)(blk / (uint32_t)p.nbx);
    const int bx = (int)(blk - (uint32_t)by * p.nbx);

    stage_window(p, ref, win32, by * p.B - p.R, bx * p.B - p.R, p.win, (p.win + 3) >> 2,
                 p.div_win4, pitch4, tid, 256);
    // current block; pixels past the frame edge (frames the block does not divide) repeat the
    // edge pixel, as the reference window does
    const bool cur_vec = (p.W & 3) == 0;
    for (int i = tid; i < p.B * B4; i += 256) {
        const int r = i / B4, c4 = i - r * B4;
        const uint8_t *row = cur + (size_t)min(by * p.B + r, p.H - 1) * p.W;
        const int gx = bx * p.B + 4 * c4;
        uint32_t v;
        if (cur_vec && gx + 3 < p.W) {
            v = *reinterpret_cast<const uint32_t *>(row + gx);
        } else {
            v = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) v |= (uint32_t)row[min(gx + b, p.W - 1)] << (8 * b);
        }
        cur32[i] = v;
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
// Row-scan kernel for 16x16 blocks and a compile-time search range R >= 8.
//
// A workgroup stages the joint search window of four horizontally adjacent
// blocks ((16+2R) rows x (64+2R) bytes); each of its four wavefronts owns one
// block.  Lane l of a wavefront owns the column of candidates dx = l - R (all
// dy).  The current block sits in 64 wave-uniform registers.  The wavefront
// walks the window rows top to bottom; for window row r a lane byte-aligns its
// 16 reference pixels once (4 x v_alignbyte) and adds them into the partial
// SADs of the (up to) sixteen candidates dy = r - i that use this row as block
// row i (4 x v_sad_u8 each), so a reference row is fetched and aligned once
// for sixteen uses.  Sixteen accumulators rotate: candidate dy completes at row
// dy + 15 and its slot restarts for dy + 16.  A lane keeps its best (sad, dy)
// as one packed key; at the end keys are widened to (sad, raster index) and
// reduced across the wavefront with DPP.
// The 2R+1 columns do not fill whole wavefronts: what is left after the full
// 64-column chunks is either run as one more (partly idle) chunk or, when it is
// narrow, one candidate per lane.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void load_aligned16(const uint32_t *rowp, uint32_t sh, uint32_t (&r)[4])
{
    const uint32_t d0 = rowp[0], d1 = rowp[1], d2 = rowp[2], d3 = rowp[3], d4 = rowp[4];
    r[0] = __builtin_amdgcn_alignbyte(d1, d0, sh);
    r[1] = __builtin_amdgcn_alignbyte(d2, d1, sh);
    r[2] = __builtin_amdgcn_alignbyte(d3, d2, sh);
    r[3] = __builtin_amdgcn_alignbyte(d4, d3, sh);
}

template <int R>
__global__ __launch_bounds__(256) void merit_sad_rowscan16(SadParams p, const uint8_t *__restrict__ cur,
                                                          const uint8_t *__restrict__ ref,
                                                          int32_t *__restrict__ sad, int32_t *__restrict__ mv)
{
    static_assert(R >= 8 && R <= 63, "steady state needs 2R >= 15");
    constexpr int N = 2 * R + 1, ROWS = 16 + 2 * R;
    constexpr int NLEFT0 = N % 64;
    constexpr bool LEFT_AS_CHUNK = NLEFT0 * N > 640;
    constexpr int NCHUNK = N / 64 + ((LEFT_AS_CHUNK && NLEFT0) ? 1 : 0);
    constexpr int NLEFT = LEFT_AS_CHUNK ? 0 : NLEFT0;
    constexpr int NS = 2 * R - 14, NSB = NS / 16, NSR = NS % 16;   // rows 15..2R use all 16 block rows

    extern __shared__ __align__(16) uint32_t lds32[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pitch4 = p.pitch >> 2;
    const uint32_t g = xcd_band_item(blockIdx.x, p.xq, p.xr);     // a band of block rows per XCD
    const int by = (int)(g / (uint32_t)p.groups_x);
    const int bx0 = (int)(g - (uint32_t)by * p.groups_x) * 4;

    stage_window(p, ref, lds32, by * 16 - R, bx0 * 16 - R, ROWS, pitch4 - 1, p.div_win4, pitch4, tid, 256);
    __syncthreads();
    const int bx = bx0 + wv;
    if (bx >= p.nbx) return;                       // ragged last group (no barrier follows)

    // current block: wave-uniform loads
    uint32_t c[16][4];
    {
        // rows past the last one (H % 16 != 0) repeat it; dwords past the end of a row
        // (W % 16 != 0, W % 4 == 0) are four copies of its last pixel
        const uint32_t *cp = reinterpret_cast<const uint32_t *>(cur);
        const int W4 = p.W >> 2;
        if ((p.W & 15) == 0) {                       // whole blocks per row: the plain loads
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = min(by * 16 + i, p.H - 1);
#pragma unroll
                for (int j = 0; j < 4; ++j) c[i][j] = cp[row * W4 + bx * 4 + j];
            }
        } else {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int row = min(by * 16 + i, p.H - 1);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int d = bx * 4 + j;
                    const uint32_t v = cp[row * W4 + min(d, W4 - 1)];
                    c[i][j] = d < W4 ? v : (v >> 24) * 0x01010101u;
                }
            }
        }
    }

    // row (lane & 15) of the current block in vector registers, for the split tail below
    // (requested here, used after the row scan)
    uint32_t crow[4];
    {
        const uint32_t *cp = reinterpret_cast<const uint32_t *>(cur);
        const int W4 = p.W >> 2;
        const int row = min(by * 16 + (lane & 15), p.H - 1);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int d = bx * 4 + j;
            const uint32_t v = cp[row * W4 + min(d, W4 - 1)];
            crow[j] = d < W4 ? v : (v >> 24) * 0x01010101u;
        }
    }

    uint32_t best = 0xffffffffu;                   // (sad << 14) | raster index
#pragma unroll 1
    for (int ch = 0; ch < NCHUNK; ++ch) {
        const int dxi = ch * 64 + lane;
        const int o = 16 * wv + min(dxi, N - 1);   // idle lanes repeat the last column
        const uint32_t sh = (uint32_t)(o & 3);
        const uint32_t *base = lds32 + (o >> 2);
        uint32_t acc[16];
#pragma unroll
        for (int k = 0; k < 16; ++k) acc[k] = 0;
        uint32_t lbest = 0xffffffffu;              // (sad << 7) | (dy + R)

        // one window row: block rows i in [ilo, ihi] accumulate into slot (rot - i) & 15;
        // then candidate `fin` (if >= 0), which sits in slot (rot + 1) & 15, is complete
        auto step = [&](const uint32_t *rowp, int ilo, int ihi, int rot, int fin) __attribute__((always_inline)) {
            uint32_t r4[4];
            load_aligned16(rowp, sh, r4);
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                if (i < ilo || i > ihi) continue;
                const int slot = (rot - i) & 15;
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[slot] = __builtin_amdgcn_sad_u8(c[i][j], r4[j], acc[slot]);
            }
            if (fin >= 0) {
                const int slot = (rot + 1) & 15;
                const uint32_t key = (acc[slot] << 7) | (uint32_t)fin;
                lbest = key < lbest ? key : lbest;
                acc[slot] = 0;
            }
        };

#pragma unroll
        for (int r = 0; r < 15; ++r) step(base + r * pitch4, 0, r, r, -1);
#pragma unroll 1
        for (int k = 0; k < NSB; ++k) {
            const uint32_t *rp = base + (15 + 16 * k) * pitch4;
#pragma unroll
            for (int j = 0; j < 16; ++j) step(rp + j * pitch4, 0, 15, (15 + j) & 15, 16 * k + j);
        }
#pragma unroll
        for (int j = 0; j < NSR; ++j)
            step(base + (15 + 16 * NSB + j) * pitch4, 0, 15, (15 + j) & 15, 16 * NSB + j);
#pragma unroll
        for (int e = 1; e <= 15; ++e)
            step(base + (2 * R + e) * pitch4, e, 15, (2 * R + e) & 15, 2 * R + e - 15);

        if (dxi < N) {
            const uint32_t dyi = lbest & 127u;
            const uint32_t key = ((lbest >> 7) << KEY_SHIFT) | (dyi * (uint32_t)N + (uint32_t)dxi);
            best = key < best ? key : best;
        }
    }

    if (NLEFT > 0) {
        // the last NLEFT columns, one candidate per lane; what does not fill a pass of 64
        // (one candidate at R = 32) is split sixteen lanes per candidate, a block row each
        constexpr int NCAND = NLEFT * N;
        constexpr int REM = NCAND % 64;
        constexpr bool SPLIT = REM > 0 && REM <= 4;
        constexpr int NFULL = SPLIT ? NCAND - REM : NCAND;
#pragma unroll 1
        for (int c0 = 0; c0 < NFULL; c0 += 64) {
            const int cand = min(c0 + lane, NCAND - 1);
            const int dyi = cand / NLEFT;
            const int dxi = (N / 64) * 64 + (cand - dyi * NLEFT);
            const int o = 16 * wv + dxi;
            const uint32_t sh = (uint32_t)(o & 3);
            const uint32_t *base = lds32 + dyi * pitch4 + (o >> 2);
            uint32_t a = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                uint32_t r4[4];
                load_aligned16(base + i * pitch4, sh, r4);
#pragma unroll
                for (int j = 0; j < 4; ++j) a = __builtin_amdgcn_sad_u8(c[i][j], r4[j], a);
            }
            const uint32_t key = (a << KEY_SHIFT) | (uint32_t)(dyi * N + dxi);
            best = key < best ? key : best;        // idle lanes recompute the last candidate
        }
        if (SPLIT) {
            const int i = lane & 15;
            const int cand = min(NFULL + (lane >> 4), NCAND - 1);
            const int dyi = cand / NLEFT;
            const int dxi = (N / 64) * 64 + (cand - dyi * NLEFT);
            const int o = 16 * wv + dxi;
            uint32_t r4[4];
            load_aligned16(lds32 + (dyi + i) * pitch4 + (o >> 2), (uint32_t)(o & 3), r4);
            uint32_t a = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) a = __builtin_amdgcn_sad_u8(crow[j], r4[j], a);
            a = group_sum_u32<16>(a);
            const uint32_t key = (a << KEY_SHIFT) | (uint32_t)(dyi * N + dxi);
            if (i == 15 && NFULL + (lane >> 4) < NCAND) best = key < best ? key : best;
        }
    }

    best = wave_min_u32(best);
    if (lane == 0) {
        const uint32_t blk = (uint32_t)by * p.nbx + bx;
        const uint32_t cidx = best & KEY_MASK;
        const int dyi = (int)(cidx / (uint32_t)N);
        sad[blk] = (int32_t)(best >> KEY_SHIFT);
        mv[2 * blk + 0] = dyi - R;
        mv[2 * blk + 1] = (int)cidx - dyi * N - R;
    }
}

// ---------------------------------------------------------------------------
// Row-scan kernel, two blocks per wavefront: for search ranges whose 2R+1 candidate columns
// fill only half a wavefront (R <= 19), each 32-lane half owns one block, so a workgroup
// covers eight horizontally adjacent blocks.  The walk over the window rows is the one
// described above with B block rows and B rotating accumulators; the current block lives
// in vector registers (it differs between the halves).  Columns beyond the 32nd are run
// one candidate per lane.  B = 8 or 16.
// ---------------------------------------------------------------------------
template <int B4>
__device__ __forceinline__ void load_aligned_row(const uint32_t *rowp, uint32_t sh, uint32_t (&r)[B4])
{
    uint32_t d[B4 + 1];
#pragma unroll
    for (int j = 0; j <= B4; ++j) d[j] = rowp[j];
#pragma unroll
    for (int j = 0; j < B4; ++j) r[j] = __builtin_amdgcn_alignbyte(d[j + 1], d[j], sh);
}

// min over each 32-lane half of a wavefront; valid in lanes 31 and 63
__device__ __forceinline__ uint32_t half_wave_min_u32(uint32_t v)
{
    v = dpp_min_step<0xB1, 0xf>(v);    // quad_perm [1,0,3,2]
    v = dpp_min_step<0x4E, 0xf>(v);    // quad_perm [2,3,0,1]
    v = dpp_min_step<0x141, 0xf>(v);   // row_half_mirror
    v = dpp_min_step<0x140, 0xf>(v);   // row_mirror: every lane holds its row's min
    v = dpp_min_step<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
    return v;
}

template <int B, int R>
__global__ __launch_bounds__(256) void merit_sad_rowscan_pair(SadParams p, const uint8_t *__restrict__ cur,
                                                             const uint8_t *__restrict__ ref,
                                                             int32_t *__restrict__ sad, int32_t *__restrict__ mv)
{
    static_assert(B == 8 || B == 16, "accumulator rotation needs a power of two");
    static_assert(2 * R >= B - 1 && 2 * R + 1 <= 40, "steady state needs 2R >= B-1; at most 8 extra columns");
    constexpr int N = 2 * R + 1, ROWS = B + 2 * R, B4 = B / 4;
    constexpr int NMAIN = N < 32 ? N : 32;          // candidate columns that are lane columns
    constexpr int NLEFT = N - NMAIN;                // the rest: one candidate per lane
    constexpr int NS = 2 * R - B + 2, NSB = NS / B, NSR = NS % B;   // rows B-1 .. 2R use all B block rows

    extern __shared__ __align__(16) uint32_t lds32[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, l32 = lane & 31, hb = lane >> 5;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int pitch4 = p.pitch >> 2;
    const uint32_t g = xcd_band_item(blockIdx.x, p.xq, p.xr);     // a band of block rows per XCD
    const int by = (int)(g / (uint32_t)p.groups_x);
    const int bx0 = (int)(g - (uint32_t)by * p.groups_x) * 8;

    stage_window(p, ref, lds32, by * B - R, bx0 * B - R, ROWS, pitch4 - 1, p.div_win4, pitch4, tid, 256);
    __syncthreads();
    const int bxl = 2 * wv + hb;                    // block inside the workgroup's window
    const int bx = bx0 + bxl;
    const bool live = bx < p.nbx;                   // ragged last group: the half computes, nothing is written

    uint32_t c[B][B4];
    {
        // rows past the last one (H % B != 0) repeat it; dwords past the end of a row
        // (W % B != 0, W % 4 == 0) are four copies of its last pixel
        const uint32_t *cp = reinterpret_cast<const uint32_t *>(cur);
        const int W4 = p.W >> 2;
        const int d0 = min(bx, p.nbx - 1) * B4;
        if ((p.W & (B - 1)) == 0) {                  // whole blocks per row: the plain loads
#pragma unroll
            for (int i = 0; i < B; ++i) {
                const int row = min(by * B + i, p.H - 1);
#pragma unroll
                for (int j = 0; j < B4; ++j) c[i][j] = cp[row * W4 + d0 + j];
            }
        } else {
#pragma unroll
            for (int i = 0; i < B; ++i) {
                const int row = min(by * B + i, p.H - 1);
#pragma unroll
                for (int j = 0; j < B4; ++j) {
                    const uint32_t v = cp[row * W4 + min(d0 + j, W4 - 1)];
                    c[i][j] = d0 + j < W4 ? v : (v >> 24) * 0x01010101u;
                }
            }
        }
    }

    // row (lane & (B-1)) of this half's current block, for the split tail below
    uint32_t crow[B4];
    {
        const uint32_t *cp = reinterpret_cast<const uint32_t *>(cur);
        const int W4 = p.W >> 2;
        const int row = min(by * B + (l32 & (B - 1)), p.H - 1);
        const int d0 = min(bx, p.nbx - 1) * B4;
#pragma unroll
        for (int j = 0; j < B4; ++j) {
            const uint32_t v = cp[row * W4 + min(d0 + j, W4 - 1)];
            crow[j] = d0 + j < W4 ? v : (v >> 24) * 0x01010101u;
        }
    }

    uint32_t best = 0xffffffffu;                    // (sad << 14) | raster index
    {
        const int dxi = l32;
        const int o = B * bxl + min(dxi, NMAIN - 1);          // idle lanes repeat the last column
        const uint32_t sh = (uint32_t)(o & 3);
        const uint32_t *base = lds32 + (o >> 2);
        uint32_t acc[B];
#pragma unroll
        for (int k = 0; k < B; ++k) acc[k] = 0;
        uint32_t lbest = 0xffffffffu;               // (sad << 7) | (dy + R)

        auto step = [&](const uint32_t *rowp, int ilo, int ihi, int rot, int fin) __attribute__((always_inline)) {
            uint32_t r4[B4];
            load_aligned_row<B4>(rowp, sh, r4);
#pragma unroll
            for (int i = 0; i < B; ++i) {
                if (i < ilo || i > ihi) continue;
                const int slot = (rot - i) & (B - 1);
#pragma unroll
                for (int j = 0; j < B4; ++j) acc[slot] = __builtin_amdgcn_sad_u8(c[i][j], r4[j], acc[slot]);
            }
            if (fin >= 0) {
                const int slot = (rot + 1) & (B - 1);
                const uint32_t key = (acc[slot] << 7) | (uint32_t)fin;
                lbest = key < lbest ? key : lbest;
                acc[slot] = 0;
            }
        };

#pragma unroll
        for (int r = 0; r < B - 1; ++r) step(base + r * pitch4, 0, r, r, -1);
#pragma unroll 1
        for (int k = 0; k < NSB; ++k) {
            const uint32_t *rp = base + (B - 1 + B * k) * pitch4;
#pragma unroll
            for (int j = 0; j < B; ++j) step(rp + j * pitch4, 0, B - 1, (B - 1 + j) & (B - 1), B * k + j);
        }
#pragma unroll
        for (int j = 0; j < NSR; ++j)
            step(base + (B - 1 + B * NSB + j) * pitch4, 0, B - 1, (B - 1 + j) & (B - 1), B * NSB + j);
#pragma unroll
        for (int e = 1; e <= B - 1; ++e)
            step(base + (2 * R + e) * pitch4, e, B - 1, (2 * R + e) & (B - 1), 2 * R + e - (B - 1));

        if (dxi < NMAIN) {
            const uint32_t dyi = lbest & 127u;
            best = ((lbest >> 7) << KEY_SHIFT) | (dyi * (uint32_t)N + (uint32_t)dxi);
        }
    }

    if (NLEFT > 0) {
        // what does not fill a pass of 32 candidates (one candidate at N = 33) is split B
        // lanes per candidate, a block row each
        constexpr int NCAND = NLEFT * N;
        constexpr int REM = NCAND % 32;
        constexpr bool SPLIT = REM > 0 && REM <= 32 / B;
        constexpr int NFULL = SPLIT ? NCAND - REM : NCAND;
#pragma unroll 1
        for (int c0 = 0; c0 < NFULL; c0 += 32) {
            const int cand = min(c0 + l32, NCAND - 1);         // idle lanes recompute the last candidate
            const int dyi = cand / NLEFT;
            const int dxi = NMAIN + (cand - dyi * NLEFT);
            const int o = B * bxl + dxi;
            const uint32_t sh = (uint32_t)(o & 3);
            const uint32_t *base = lds32 + dyi * pitch4 + (o >> 2);
            uint32_t a = 0;
#pragma unroll
            for (int i = 0; i < B; ++i) {
                uint32_t r4[B4];
                load_aligned_row<B4>(base + i * pitch4, sh, r4);
#pragma unroll
                for (int j = 0; j < B4; ++j) a = __builtin_amdgcn_sad_u8(c[i][j], r4[j], a);
            }
            const uint32_t key = (a << KEY_SHIFT) | (uint32_t)(dyi * N + dxi);
            best = key < best ? key : best;
        }
        if (SPLIT) {
            const int i = l32 & (B - 1);
            const int ci = NFULL + l32 / B;
            const int cand = min(ci, NCAND - 1);
            const int dyi = cand / NLEFT;
            const int dxi = NMAIN + (cand - dyi * NLEFT);
            const int o = B * bxl + dxi;
            uint32_t r4[B4];
            load_aligned_row<B4>(lds32 + (dyi + i) * pitch4 + (o >> 2), (uint32_t)(o & 3), r4);
            uint32_t a = 0;
#pragma unroll
            for (int j = 0; j < B4; ++j) a = __builtin_amdgcn_sad_u8(crow[j], r4[j], a);
            a = group_sum_u32<B>(a);
            const uint32_t key = (a << KEY_SHIFT) | (uint32_t)(dyi * N + dxi);
            if (i == B - 1 && ci < NCAND) best = key < best ? key : best;
        }
    }

    best = half_wave_min_u32(best);
    if (l32 == 31 && live) {
        const uint32_t blk = (uint32_t)by * p.nbx + bx;
        const uint32_t cidx = best & KEY_MASK;
        const int dyi = (int)(cidx / (uint32_t)N);
        sad[blk] = (int32_t)(best >> KEY_SHIFT);
        mv[2 * blk + 0] = dyi - R;
        mv[2 * blk + 1] = (int)cidx - dyi * N - R;
    }
}

// ---------------------------------------------------------------------------
hipError_t launch_sad(const SadParams &p, const uint8_t *cur, const uint8_t *ref, int32_t *sad,
                      int32_t *mv, hipStream_t s)
{
    const uint32_t nblocks = (uint32_t)(p.nby * p.nbx);
    if (nblocks == 0) return hipSuccess;
    const int pitch4 = p.pitch >> 2;
    if (p.variant == SAD_ROWSCAN_B16) {
        const uint32_t grid = (uint32_t)(p.nby * p.groups_x);
        const size_t lds_bytes = (size_t)((16 + 2 * p.R) * pitch4 + 1) * 4;
        if (p.R == 32)
            hipLaunchKernelGGL(merit_sad_rowscan16<32>, dim3(grid), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
        else
            hipLaunchKernelGGL(merit_sad_rowscan16<16>, dim3(grid), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
        return hipGetLastError();
    }
    if (p.variant == SAD_ROWSCAN_PAIR) {
        const uint32_t grid = (uint32_t)(p.nby * p.groups_x);
        const size_t lds_bytes = (size_t)((p.B + 2 * p.R) * pitch4 + 1) * 4;
        if (p.B == 8 && p.R == 16)
            hipLaunchKernelGGL((merit_sad_rowscan_pair<8, 16>), dim3(grid), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
        else if (p.B == 8 && p.R == 8)
            hipLaunchKernelGGL((merit_sad_rowscan_pair<8, 8>), dim3(grid), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
        else if (p.B == 16 && p.R == 16)
            hipLaunchKernelGGL((merit_sad_rowscan_pair<16, 16>), dim3(grid), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
        else
            return hipErrorInvalidValue;
        return hipGetLastError();
    }
    const size_t lds_bytes = (size_t)(p.win * pitch4 + 1 + p.B * (p.B >> 2) + 4) * 4;
    hipLaunchKernelGGL(merit_sad_generic, dim3(nblocks), dim3(256), lds_bytes, s, p, cur, ref, sad, mv);
    return hipGetLastError();
}

const char *sad_kernel_name(const SadParams &p)
{
    if (p.variant == SAD_ROWSCAN_B16) return p.R == 32 ? "merit_sad_rowscan16<32>" : "merit_sad_rowscan16<16>";
    if (p.variant == SAD_ROWSCAN_PAIR)
        return p.B == 16 ? "merit_sad_rowscan_pair<16,16>" : (p.R == 16 ? "merit_sad_rowscan_pair<8,16>" : "merit_sad_rowscan_pair<8,8>");
    return "merit_sad_generic";
}

}  // namespace merit
