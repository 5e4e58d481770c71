// Correlation layer for gfx950 (Section III-C, Eq. 8):
//     M(I1)[p,a] = I1[b, a1, p1, p2]
//     M(I2)[p,a] = I2[b, a1, p1 + (p3-R)*sd, p2 + (p4-R)*sd]      (0 outside the image)
// with k = (b, p1, p2, p3, p4 | a1) and the dot product over the channel index a1
// (Section III-B, Eq. 3).  Output y[b,p1,p2,p3,p4], binary16, fp32 accumulation.
//
// A workgroup owns (b, p1, p3, a run of 64 pixels p2): one row of the first tensor and one
// (displaced) row of the second.  For that pair of rows the layer is a banded matrix product:
// with the pixels p2 as rows, the columns q of the second row as columns and the channels as
// the reduction axis, D = X1^T X2 holds y[.., p2, p3, p4] at q = p2 + (p4-R)*sd.  Only columns
// congruent to p2 modulo sd are ever needed, so a block of 16 pixels of one residue class is
// multiplied with the 16+2R columns of the same class around it, in blocks of 16
// (v_mfma_f32_16x16x32_f16, a third of the products are wanted ones at R = 5); the matrix
// cores do in a few hundred cycles what the vector dot products took most of the kernel for.
// Both rows are staged in LDS with the channel axis innermost, eight channels = 16 bytes per
// pixel, transposed in registers on the way (v_perm_b32): exactly the operand a lane feeds to
// the MFMA.  Positions are ordered by residue class so that the 16 pixels of a block are
// adjacent.  Channels go through LDS in passes of `chg` groups of eight; the loads of the next
// pass are in flight while the current one is multiplied.  Needs W % 8 == 0, R <= 15, sd <= 8.
#include "merit_internal.h"

namespace merit {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int XB = CORR_XB;    // staging units a thread holds in registers per pass

// One staging unit = 8 adjacent pixels x 8 channels of one row: eight 16-byte loads (one per
// channel), transposed to eight 16-byte LDS items (one per pixel).  The units of a pass form
// one list: for each channel group the chunk's units of the first tensor, then those of the
// second.  8-column units outside the row (starts are multiples of 8, W % 8 == 0) and
// missing channels give zeros.
struct StageGeom {
    int b, p1, yy, px0, npx8, gx2;
    uint32_t per_g;
    FastDiv div_perg;
};

__device__ __forceinline__ void issue_pass(const CorrParams &p, const StageGeom &sg,
                                           const uint16_t *__restrict__ x1, const uint16_t *__restrict__ x2,
                                           int chi0, int ng, int tid, uint32_t (&v)[XB][8][4])
{
    const uint32_t nu = (uint32_t)ng * sg.per_g;
    const size_t chstride = (size_t)p.H * p.W;
#pragma unroll
    for (int k = 0; k < XB; ++k) {
        const uint32_t u = min((uint32_t)tid + 256u * k, nu - 1);
        const uint32_t g = fdiv(u, sg.div_perg);
        const int r = (int)(u - g * sg.per_g);
        const bool second = r >= sg.npx8;
        const int gx = second ? sg.gx2 + 8 * (r - sg.npx8) : sg.px0 + 8 * r;
        const int gy = second ? sg.yy : sg.p1;
        const bool colok = gx >= 0 && gx < p.W;
        const int c0 = (chi0 + (int)g) * 8;
        const uint16_t *xs = second ? x2 : x1;
        const uint16_t *src = xs + (((size_t)sg.b * p.C + min(c0, p.C - 1)) * p.H + gy) * p.W + (colok ? gx : 0);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const bool ok = colok && (c0 + c < p.C);
            // branch-free: a missing element re-reads the tensor's first bytes and is zeroed
            const uint4 t4 = *reinterpret_cast<const uint4 *>(ok ? src + c * chstride : xs);
            v[k][c][0] = ok ? t4.x : 0u; v[k][c][1] = ok ? t4.y : 0u;
            v[k][c][2] = ok ? t4.z : 0u; v[k][c][3] = ok ? t4.w : 0u;
        }
    }
}

__device__ __forceinline__ void commit_pass(const CorrParams &p, const StageGeom &sg, uint4 *a1l, uint4 *a2l,
                                            int ng, int tid, const uint32_t (&v)[XB][8][4])
{
    const uint32_t nu = (uint32_t)ng * sg.per_g;
#pragma unroll
    for (int k = 0; k < XB; ++k) {
        const uint32_t u = (uint32_t)tid + 256u * k;
        if (u >= nu) break;
        const uint32_t g = fdiv(u, sg.div_perg);
        const int r = (int)(u - g * sg.per_g);
        const bool second = r >= sg.npx8;
        const int run = second ? r - sg.npx8 : r;
        uint4 *d4 = second ? a2l + g * p.P2 : a1l + g * p.P1;
        const int pitch = second ? p.pitch2 : p.pitch1;
#pragma unroll
        for (int px = 0; px < 8; ++px) {
            const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
            uint32_t d[4];
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                d[qq] = __builtin_amdgcn_perm(v[k][2 * qq + 1][px >> 1], v[k][2 * qq][px >> 1], sel);
            const uint32_t col = (uint32_t)(8 * run + px);
            const uint32_t idx = fdiv(col, p.div_sd);
            const uint32_t cls = col - idx * (uint32_t)p.sd;
            d4[cls * (uint32_t)pitch + idx] = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
}

// NB = 16-column blocks of the second row per pixel block, BPW = pixel blocks per wavefront.
template <int NB, int BPW>
__global__ __launch_bounds__(256, 4) void merit_corr_mfma(CorrParams p, const uint16_t *__restrict__ x1,
                                                       const uint16_t *__restrict__ x2, uint16_t *__restrict__ y)
{
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *a1l = reinterpret_cast<uint4 *>(smem);                 // [chg][P1]
    uint4 *a2l = a1l + p.chg * p.P1;                              // [chg][P2]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // each XCD takes a band of image rows: its L2 then fetches that band and its halo rows of
    // the second tensor, not both whole tensors
    uint32_t g = xcd_band_item(blockIdx.x, p.xq, p.xr);
    // work item -> (b, p1, p3, pixel chunk), chunk fastest
    const uint32_t q0 = fdiv(g, p.div_xchunks);
    const int xc = (int)(g - q0 * (uint32_t)p.xchunks);
    const uint32_t q1 = fdiv(q0, p.div_n);
    const int p3 = (int)(q0 - q1 * (uint32_t)p.n);
    const int b = (int)fdiv(q1, p.div_h);
    const int p1 = (int)(q1 - (uint32_t)b * (uint32_t)p.H);

    StageGeom sg;
    sg.b = b; sg.p1 = p1; sg.px0 = xc * 64;
    sg.yy = p1 + (p3 - p.R) * p.sd;
    sg.npx8 = min(8, (p.W - sg.px0) >> 3);                        // 8-pixel units of the first tensor's chunk
    sg.gx2 = sg.px0 - p.lead;                                     // first staged column of the second tensor
    sg.per_g = (uint32_t)(sg.npx8 + (p.cols2 >> 3));
    sg.div_perg = sg.npx8 == 8 ? p.div_perg : p.div_perg_last;
    const bool rowok = sg.yy >= 0 && sg.yy < p.H;
    const int wchunk = min(64, p.W - sg.px0);                     // pixels of this chunk

    // this lane's operand positions: pixel (lane & 15) of block (class c, sub-block s) and the
    // columns q = pixel0 - R*sd + sd*j of the same class, j = 16*nb + (lane & 15); positions
    // past the staged ones are clamped (their products are never stored)
    const int l16 = lane & 15, kg = lane >> 4;
    int apos[BPW], bpos[BPW][NB];
#pragma unroll
    for (int t = 0; t < BPW; ++t) {
        const uint32_t bl = (uint32_t)min(wave + 4 * t, p.nblk - 1);
        const uint32_t s = fdiv(bl, p.div_sd);
        const uint32_t c = bl - s * (uint32_t)p.sd;
        apos[t] = min((int)c * p.pitch1 + 16 * (int)s + l16, p.P1 - 1);
        const uint32_t ec = (uint32_t)(p.lead - p.R * p.sd) + c;
        const uint32_t ei = fdiv(ec, p.div_sd);
        const uint32_t cls2 = ec - ei * (uint32_t)p.sd;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
            bpos[t][nb] = min((int)cls2 * p.pitch2 + (int)ei + 16 * (int)s + 16 * nb + l16, p.P2 - 1);
    }

    floatx4 acc[BPW][NB];
#pragma unroll
    for (int t = 0; t < BPW; ++t)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) acc[t][nb] = floatx4{0.0f, 0.0f, 0.0f, 0.0f};

    if (rowok) {                                                  // uniform: else every product is 0
        // groups of the pass that starts at chi0, padded to whole reduction steps (the padding is staged as zeros)
        auto groups_of = [&](int chi0) { return min(p.chg, ((p.nchi - chi0) + 3) & ~3); };
        uint32_t v[XB][8][4];
        issue_pass(p, sg, x1, x2, 0, groups_of(0), tid, v);
        for (int chi0 = 0; chi0 < p.nchi; chi0 += p.chg) {
            const int ng = groups_of(chi0);
            if (chi0 > 0) __syncthreads();                        // previous pass has been read
            commit_pass(p, sg, a1l, a2l, ng, tid, v);
            __syncthreads();
            // the next pass's loads are in flight while this one is multiplied
            const int nxt = chi0 + p.chg;
            if (nxt < p.nchi) issue_pass(p, sg, x1, x2, nxt, groups_of(nxt), tid, v);
#pragma unroll
            for (int t = 0; t < BPW; ++t) {
                if (wave + 4 * t >= p.nblk) break;                // uniform
                const uint4 *ap = a1l + kg * p.P1 + apos[t];
                const uint4 *bp = a2l + kg * p.P2;
                for (int ks = 0; ks < ng; ks += 4) {
                    const half8 a = __builtin_bit_cast(half8, ap[ks * p.P1]);
                    half8 bq[NB];
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb) bq[nb] = __builtin_bit_cast(half8, bp[ks * p.P2 + bpos[t][nb]]);
#pragma unroll
                    for (int nb = 0; nb < NB; ++nb)
                        acc[t][nb] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq[nb], acc[t][nb], 0, 0, 0);
                }
            }
        }
    }

    // D[i][j]: lane holds column j = lane & 15 and rows i = 4*(lane >> 4) + r.  Row i is pixel
    // i of the block, column 16*nb + j is displacement p4 = 16*nb + j - i.
    uint16_t *yrow = y + (((size_t)b * p.H + p1) * p.W + sg.px0) * p.n * p.n + (size_t)p3 * p.n;
#pragma unroll
    for (int t = 0; t < BPW; ++t) {
        const int bl = wave + 4 * t;
        if (bl >= p.nblk) break;                                  // uniform
        const uint32_t s = fdiv((uint32_t)bl, p.div_sd);
        const int c = bl - (int)s * p.sd;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = 4 * kg + r;
            const int px = c + p.sd * (16 * (int)s + i);          // pixel inside the chunk
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const int p4 = 16 * nb + l16 - i;
                if (px < wchunk && p4 >= 0 && p4 < p.n) {
                    const _Float16 h = (_Float16)acc[t][nb][r];   // round to nearest even
                    yrow[(size_t)px * p.n * p.n + p4] = __builtin_bit_cast(uint16_t, h);
                }
            }
        }
    }
}

size_t corr_lds_bytes(const CorrParams &p)
{
    return (size_t)p.chg * (p.P1 + p.P2) * 16;
}

template <int NB, int BPW>
static hipError_t launch_corr(const CorrParams &p, const void *x1, const void *x2, void *y, hipStream_t s,
                              uint32_t grid)
{
    static std::atomic<int> raised{0};
    if (hipError_t e = raise_lds_limit_once(reinterpret_cast<const void *>(merit_corr_mfma<NB, BPW>), raised);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((merit_corr_mfma<NB, BPW>), dim3(grid), dim3(256), corr_lds_bytes(p), s, p,
                       reinterpret_cast<const uint16_t *>(x1), reinterpret_cast<const uint16_t *>(x2),
                       reinterpret_cast<uint16_t *>(y));
    return hipGetLastError();
}

hipError_t launch_correlation(const CorrParams &p, const void *x1, const void *x2, void *y, hipStream_t s)
{
    const int64_t grid = (int64_t)p.N * p.H * p.n * p.xchunks;
    if (grid == 0) return hipSuccess;
    const uint32_t gx = (uint32_t)grid;
    const int bpw = (p.nblk + 3) / 4;
    if (bpw < 1 || bpw > 2) return hipErrorInvalidValue;
    switch (p.nb * 2 + (bpw - 1)) {
    case 2: return launch_corr<1, 1>(p, x1, x2, y, s, gx);
    case 3: return launch_corr<1, 2>(p, x1, x2, y, s, gx);
    case 4: return launch_corr<2, 1>(p, x1, x2, y, s, gx);
    case 5: return launch_corr<2, 2>(p, x1, x2, y, s, gx);
    case 6: return launch_corr<3, 1>(p, x1, x2, y, s, gx);
    case 7: return launch_corr<3, 2>(p, x1, x2, y, s, gx);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace merit
