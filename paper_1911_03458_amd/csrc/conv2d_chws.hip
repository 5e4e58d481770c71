// 2-D convolution for gfx950, many input channels: wave-specialised, double-buffered passes.
//
// k = (n, co, oy, ox | ci, ky, kx) (Section III-C, Eq. 6), reduced with the dot product
// (Section III-B, Eq. 3) on v_mfma_f32_32x32x16_f16, K order (ci/8, ky, kx | ci%8) as in the
// channel-block kernels of conv2d.hip.  What differs is who does what and how large a
// wavefront's register tile is:
//
//   * A workgroup is 8 wavefronts.  Wavefronts 0-3 only multiply: each owns PXB x CHB blocks of
//     32 pixels x 32 output channels (128 x 64 by default), so a K step reads PXB + CHB
//     fragments from LDS for PXB * CHB MFMAs (6 reads per 8 MFMAs instead of 3 per 2), and the
//     reads of step s+1 are issued before the MFMAs of step s.
//   * Wavefronts 4-7 only move data.  The input channels go through LDS in passes of 16 (two
//     groups of 8, one per half of a wavefront); pass q+1 is transposed into the other LDS
//     buffer while pass q is multiplied, and the global loads of passes q+2 and q+3 are in
//     flight meanwhile (two register sets).  One barrier per pass.
//   * The covering sub-tensor of a tile (Section IV-A, Eq. 9) is TM consecutive output pixels
//     of one image (whole rows: only a vertical halo) x 16 channels per pass.
//
// Weights are either the caller's [Cout][Cin][kh][kw] tensor, transposed in registers by the
// moving wavefronts on every pass, or a buffer that merit_conv2d_pack_weights wrote once in
// exactly the order the passes want them (then a pass's weights are one contiguous copy).
#include "merit_internal.h"

#include <atomic>
#include <mutex>

namespace merit {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint32x2 __attribute__((ext_vector_type(2)));

union Frag {
    uint4 u;
    half8 h;
};

struct Geom {
    int n, m0, oyA, yA, RH, cg;
    int mend;      // one past the last output pixel of the tile that is used
    // fused pooling only
    int pr0;       // first pooled row the tile completes
    int warm;      // the tile above a band's first pooled row: only its last row is kept
    int top;       // the tile starts at the image's first row: nothing above it (-inf)
    int roff;      // row of the tile that is convolution row 2 pr0 (1 when the tile computes the row above it)
    int par;       // which of the two carry buffers holds the row above the tile
};

__device__ __forceinline__ Geom tile_geom(const ConvParams &p, int item, int ohw)
{
    Geom g;
    const int tile = (int)fdiv((uint32_t)item, p.div_cog);
    g.cg = item - tile * p.co_groups;
    g.n = (int)fdiv((uint32_t)tile, p.div_tiles);
    g.m0 = (tile - g.n * p.tiles_per_image) * p.tile_px;
    g.oyA = (int)fdiv((uint32_t)g.m0, p.div_ow);
    const int mlast = min(g.m0 + p.tile_px, ohw) - 1;
    const int oyB = (int)fdiv((uint32_t)mlast, p.div_ow);
    g.yA = g.oyA * p.sh - p.ph;
    g.RH = p.row_skip ? oyB - g.oyA + 1 : (oyB - g.oyA) * p.sh + (p.kh - 1) * p.dh + 1;
    g.mend = min(g.m0 + p.tile_px, ohw);
    g.pr0 = g.warm = g.top = g.roff = g.par = 0;
    return g;
}

// Fused 3x3 / stride 2 / padding 1 max pooling: a work item is (image, band of PB pooled rows,
// channel block); its tiles are whole convolution rows.  Pooled row r needs rows 2r-1, 2r, 2r+1.
// Two ways to get row 2r-1 for a tile's first pooled row:
//   * carried (pool_halo = 0): a tile is rows_out_max (even) rows from the even row 2 pr0 and
//     completes rows_out_max / 2 pooled rows from its own rows and the last row of the tile before
//     it, which is kept in LDS.  The first tile of a band below the image's top only produces that
//     carried row.
//   * computed (pool_halo = 1): a tile is rows_out_max (odd) rows from row 2 pr0 - 1 and completes
//     (rows_out_max - 1) / 2 pooled rows on its own; a band is one tile.
__device__ __forceinline__ int pool_band_tiles(const ConvParams &p, int item)
{
    if (p.pool_halo) return 1;
    const int bu = (int)fdiv((uint32_t)item, p.div_cog);
    const int n = (int)fdiv((uint32_t)bu, p.div_nb);
    const int band = bu - n * p.NB;
    const int rows = min(p.PB, p.PH - band * p.PB);                  // pooled rows of this band
    const int hp = p.rows_out_max >> 1;
    return (rows + hp - 1) / hp + (band > 0 ? 1 : 0);
}

__device__ __forceinline__ Geom pool_geom(const ConvParams &p, int item, int i, int ohw)
{
    Geom g;
    const int bu = (int)fdiv((uint32_t)item, p.div_cog);
    g.cg = item - bu * p.co_groups;
    g.n = (int)fdiv((uint32_t)bu, p.div_nb);
    const int band = bu - g.n * p.NB;
    const int R = p.rows_out_max, hp = R >> 1;
    const int lead = (band > 0 && !p.pool_halo) ? 1 : 0;
    g.pr0 = band * p.PB + (i - lead) * hp;                           // (the warm-up tile: hp rows higher, nothing of it is stored)
    g.warm = (lead && i == 0) ? 1 : 0;
    g.top = g.pr0 == 0 ? 1 : 0;
    g.roff = (p.pool_halo && !g.top) ? 1 : 0;
    g.oyA = 2 * g.pr0 - g.roff;
    g.par = i & 1;
    g.m0 = g.oyA * p.OW;
    g.mend = min(g.m0 + R * p.OW, ohw);
    g.yA = g.oyA * p.sh - p.ph;
    g.RH = (R - 1) * p.sh + (p.kh - 1) * p.dh + 1;
    return g;
}

constexpr int XS_MAX = 8;      // input units of 8 channels x 1 pixel a moving thread holds per pass (4 beside 8 multiplying wavefronts -- 168 registers -- and for 5x5 windows)
constexpr uint32_t OOB = 0x80000000u;   // a buffer offset past the end of every tensor: loads return zeros

}  // namespace

// PXB x CHB: 32x32 blocks per multiplying wavefront; WM x WN = 4 multiplying wavefronts.
// T: taps of the window (25 = 5x5, 9 = 3x3, 1 = 1x1).  XU = 1, 2: the input rows are staged in units of 8
// channels x 8 pixels (W % 8 == 0), XU of them per moving thread and pass; XU = 0: in units of
// 8 channels x 1 pixel, up to XS_MAX per thread.
// NG: pairs of 8-channel groups per pass (1: 16 channels, 2: 32 -- small tiles, whose passes would
// otherwise be shorter than a memory round trip; 4: 64 -- 1x1 windows on many channels).
// POOL: the results are max-pooled (3x3 / stride 2 / padding 1) out of the staging area and only the
// pooled tensor is written; work items are bands of pooled rows (pool_geom above).
// RES: a tensor of the output's shape is added to the fp32 sums before the clip and the rounding.
template <int PXB, int CHB, int WM, int WN, int T, int XU, bool PACKED, int NG = 1, bool POOL = false, bool RES = false>
__global__ __launch_bounds__((WM * WN + 4) * 64, 1) void merit_conv2d_chws(ConvParams p, const uint16_t *__restrict__ x,
                                                            const uint16_t *__restrict__ w,
                                                            const uint16_t *res, uint16_t *y)
{
    constexpr int NMW = WM * WN;                         // multiplying wavefronts; four more move data
    static_assert(NMW == 4 || NMW == 8, "one or two multiplying wavefronts per SIMD");
    constexpr int NT = (NMW + 4) * 64;                   // threads per workgroup
    constexpr int TM = WM * PXB * 32, NCB = WN * CHB, TN = NCB * 32;
    constexpr int WITEMS = NG * T * NCB * 64;            // 16-byte weight fragments per pass
    constexpr int NGRP = 2 * NG;                         // 8-channel groups per pass
    constexpr int WU = (TN * NGRP + 255) / 256;          // weight units (8 channels x T taps of one output channel) per moving thread
    constexpr int OP = TM / 2 + 2;                       // output staging: dwords per channel
    constexpr bool XV = XU == 1 || XU == 2;              // 8-pixel input units, XU per moving thread
    constexpr bool XQ = XU == 4;                         // 4-pixel input units (W % 4 == 0)
    constexpr bool XD = XU == 3;                         // 2-pixel input units (W % 4 == 2: rows start on 4-byte boundaries)

    {
        // The kernel-argument block (ConvParams and three pointers: six 64-byte lines) is read with
        // scalar loads where the values are first needed; touching every line with the very first
        // instructions fetches them side by side instead of one memory trip after the other.
        static_assert(sizeof(ConvParams) + 4 * sizeof(void *) <= 6 * 64, "six lines of kernel arguments");
        typedef const uint32_t __attribute__((address_space(4))) *kernarg_ptr;
        kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
        const uint32_t warm = ka[0] ^ ka[16] ^ ka[32] ^ ka[48] ^ ka[64] ^ ka[80];
        asm volatile("" ::"s"(warm));
    }
    extern __shared__ __align__(16) uint8_t smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, h = lane >> 5, c32 = lane & 31;
    const bool mover = wave >= NMW;
    const int mt = tid - NMW * 64;                       // index among the moving threads
    const int ohw = p.OH * p.OW;
    const int npass = p.nchunks;

    auto wbuf = [&](int b) { return reinterpret_cast<uint4 *>(smem + b * p.lds_buf_bytes); };
    auto xbuf = [&](int b) { return reinterpret_cast<uint4 *>(smem + b * p.lds_buf_bytes + p.lds_w_bytes); };
    uint32_t *outl = reinterpret_cast<uint32_t *>(smem);

    // ---- work list: item = (tile, channel block), a contiguous band of the list per XCD ------
    const int nitems = POOL ? p.N * p.NB * p.co_groups : p.N * p.tiles_per_image * p.co_groups;
    const int stride = (int)gridDim.x;
    int item = (int)xcd_band_item(blockIdx.x, stride >> 3, stride & 7);
    if (item >= nitems) return;                            // (the launcher never makes the grid larger than the list)
    // position = (item, tile of the item); without pooling an item is one tile
    int ti = 0, ntile = POOL ? pool_band_tiles(p, item) : 1;
    auto geom_at = [&](int it, int i) __attribute__((always_inline)) {
        if constexpr (POOL) return pool_geom(p, it, i, ohw);
        else return tile_geom(p, it, ohw);
    };
    auto next_pos = [&](int &it, int &i, int &n) __attribute__((always_inline)) -> bool {
        if constexpr (POOL) {
            if (++i < n) return true;
            i = 0;
        }
        it += stride;
        if (it >= nitems) return false;
        if constexpr (POOL) n = pool_band_tiles(p, it);
        return true;
    };

    // results: LDS [channel][pixel] -> 16-byte runs along the pixel axis, by all threads
    auto store_out = [&](const Geom &g) __attribute__((always_inline)) {
        constexpr int UNITS = TN * (TM / 8);
        if ((ohw & 7) != 0) {                                // 13x13, 27x27, 7x7: planes off the 16-byte grid
            const int cnt = g.mend - g.m0;
            store_runs_on_grid<TM, NT>(outl, y, ((size_t)g.n * p.Cout + g.cg * TN) * ohw + g.m0, ohw, cnt,
                                       min(TN, p.Cout - g.cg * TN), cnt - 7, true, true, tid);
            return;
        }
#pragma unroll 4
        for (int u = tid; u < UNITS; u += NT) {
            const int c = u / (TM / 8);
            const int px8 = u - c * (TM / 8);
            const int m = g.m0 + px8 * 8;
            const int co = g.cg * TN + c;
            if (m >= g.mend || co >= p.Cout) continue;       // (a tile of whole rows ends before the 256th pixel)
            const uint2 *src = reinterpret_cast<const uint2 *>(outl + c * OP + px8 * 4);
            const uint2 lo = src[0], hi = src[1];
            uint16_t *y0 = y + ((size_t)g.n * p.Cout + co) * ohw + m;
            uint32x4 v;
            v.x = lo.x; v.y = lo.y; v.z = hi.x; v.w = hi.y;
            __builtin_nontemporal_store(v, reinterpret_cast<uint32x4 *>(y0));
        }
    };

    // Fused pooling, by all threads: unit = (channel, pooled row of the tile, 4 pooled pixels).  The
    // rows 2r-1, 2r, 2r+1 are 4 dwords (8 convolution pixels) each plus the dword to their left;
    // row -1 of the tile comes from the carry buffer the previous tile filled (-inf above the
    // image).  Maximum down the rows, then along the row at stride 2.  Before that the tile's last
    // row goes to the other carry buffer.  binary16 maxima are exact: the result is bit-equal to
    // pooling the stored convolution.
    auto pool_out = [&](const Geom &g) __attribute__((always_inline)) {
        static_assert((TN & (TN - 1)) == 0, "channel index = low bits of the unit index");
        constexpr uint32_t NINF = 0xFC00FC00u;
        const int OW2 = p.OW >> 1;                         // dwords per convolution row
        const int R = p.rows_out_max, hp = R >> 1;
        uint32_t *carry = reinterpret_cast<uint32_t *>(smem + p.lds_o_offset);
        const uint32_t *cin = carry + g.par * (TN * OW2);
        if (!p.pool_halo) {
            uint32_t *cnext = carry + (g.par ^ 1) * (TN * OW2);
            for (int u = tid; u < TN * OW2; u += NT) {
                const int c = u & (TN - 1), d = u / TN;
                cnext[c * OW2 + d] = outl[c * OP + (R - 1) * OW2 + d];
            }
            if (g.warm) return;
        }
        auto pmax = [](uint32_t a, uint32_t b) {
            return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b)));
        };
        const int units = TN * hp * p.pw8;
        const bool vec_ok = (p.PW & 3) == 0;
        for (int u = tid; u < units; u += NT) {
            const int c = u & (TN - 1), v = u / TN;
            const int prl = (int)fdiv((uint32_t)v, p.div_pw8);
            const int j4 = v - prl * p.pw8;
            const int pr = g.pr0 + prl;
            const int co = g.cg * TN + c;
            if (pr >= p.PH || co >= p.Cout) continue;
            const int rowb = g.roff + 2 * prl;                                  // the tile's row that is convolution row 2r
            const uint32_t *rb = outl + c * OP + rowb * OW2 + 4 * j4;            // row 2r; row 2r+1 is OW2 further
            const uint32_t *ra = rowb > 0 ? rb - OW2 : cin + c * OW2 + 4 * j4;   // row 2r-1: the tile's, or the carried one
            const bool above = rowb > 0 || !g.top;
            uint32_t vm[4], left;
#pragma unroll
            for (int q = 0; q < 4; ++q) vm[q] = pmax(pmax(rb[q], rb[OW2 + q]), above ? ra[q] : NINF);
            if (j4 > 0) left = pmax(pmax(rb[-1], rb[OW2 - 1]), above ? ra[-1] : NINF);
            else left = NINF;
            uint32_t res[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t prev = (k == 0 ? left : vm[k - 1]) >> 16;          // pixel 2k-1 in the low half
                res[k] = pmax(pmax(vm[k], vm[k] >> 16), prev) & 0xffffu;         // max of pixels 2k-1, 2k, 2k+1
            }
            uint16_t *y0 = y + (((size_t)g.n * p.Cout + co) * p.PH + pr) * p.PW + 4 * j4;
            if (vec_ok) {
                uint2 o;
                o.x = res[0] | (res[1] << 16);
                o.y = res[2] | (res[3] << 16);
                *reinterpret_cast<uint2 *>(y0) = o;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (4 * j4 + k < p.PW) y0[k] = (uint16_t)res[k];
            }
        }
    };

    // Both kinds of wavefront run the same sequence of barriers (npass + 3 per work item):
    //   P      pass 0 is in buffer 0
    //   B_ck   pass ck has been multiplied, pass ck+1 is in the other buffer
    //   E1     the accumulators are in the output staging area (which overlays the buffers)
    //   E2     the staging area has been stored: the buffers are free again
    if (mover) {
        // ---- the moving wavefronts ----
        // Global memory is read through buffer descriptors: a unit that lies outside the tensors
        // (rows above or below the image, padding channels of the last pass, channels past Cout)
        // gets the offset OOB and comes back as zeros: no branch and no select on the data.
        // Per-thread offsets and LDS addresses are worked out once per work item; a pass adds
        // scalar offsets only.
        const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(x), 0, (int)((size_t)p.N * p.Cin * p.H * p.W * 2), 0x00020000);
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(w), 0,
            (int)(PACKED ? (size_t)p.co_groups * npass * WITEMS * 16 : (size_t)p.Cout * p.Cin * T * 2), 0x00020000);
        const uint32_t chbytes = (uint32_t)(p.H * p.W * 2);          // one channel of one image
        const int mwave = wave - NMW;

        constexpr int XSM = (NMW == 4 && T != 25) ? XS_MAX : 4;       // (5x5: 100 registers of weights on their way)
        constexpr int XQM = NMW == 4 ? 4 : 2;                // 4-pixel units per moving thread, at most
        constexpr int XDM = XSM;                             // 2-pixel units per moving thread, at most
        constexpr int NXU = XV ? XU : (XQ ? XQM : (XD ? XDM : XSM));
        uint32_t x_voff[NXU];               // byte offset of the unit inside (image, first channel of the pass)
        int x_lds[NXU][XV ? 8 : (XQ ? 4 : (XD ? 2 : 1))];   // byte address of each of its pixels inside a pass buffer's input region
        int x_hh[NXU];                      // its channel group within the pass
        uint32_t xv[XV ? XU : 1][8][4];     // the unit on its way: 8 channels x 8 pixels
        uint32_t xs[(XV || XQ || XD) ? 1 : XSM][8];    // ... 8 channels x 1 pixel (a register each: see commit)
        uint32_t xq[XQ ? XQM : 1][8][2];         // ... 8 channels x 4 pixels
        uint32_t xd[XD ? XDM : 1][8];            // ... 8 channels x 2 pixels
        uint32_t w_voff[WU];
        int w_lds[WU], w_hh[WU];
        uint32_t wr[PACKED ? 1 : WU][PACKED ? 1 : 4 * T];

        const int rstep = p.row_skip ? p.sh : 1;        // image rows between staged rows
        auto setup = [&](const Geom &g) __attribute__((always_inline)) {
            if constexpr (XV) {
                const int W8 = p.W >> 3;
                const int nu = NGRP * p.RHa * W8;
#pragma unroll
                for (int k = 0; k < XU; ++k) {
                    // consecutive threads take consecutive staged rows (q = group * RHa + row) of one
                    // 8-pixel column chunk: their LDS writes are q * pitch items apart, and the pitch
                    // is odd, so 16 of them fall into 16 different bank groups
                    const int u = mt + 256 * k;
                    const int uc = min(u, nu - 1);
                    const int x8 = (int)fdiv((uint32_t)uc, p.div_r2);
                    const int q = uc - x8 * NGRP * p.RHa;
                    const int hh = (int)fdiv((uint32_t)q, p.div_rha);
                    const int r = q - hh * p.RHa;
                    const int gy = g.yA + r * rstep;
                    const bool ok = u < nu && r < g.RH && gy >= 0 && gy < p.H;
                    x_hh[k] = u < nu ? hh : NGRP;                            // NGRP: no such unit, never written
                    x_voff[k] = ok ? (uint32_t)(((hh * 8 * p.H + gy) * p.W + 8 * x8) * 2) : OOB;
#pragma unroll
                    for (int px = 0; px < 8; ++px)
                        x_lds[k][px] = (q * p.pitch + p.padl + 8 * x8 + px) * 16;
                }
            } else if constexpr (XQ) {
                const int W4 = p.W >> 2;
                const int nu = NGRP * p.RHa * W4;
#pragma unroll
                for (int k = 0; k < XQM; ++k) {
                    const int u = mt + 256 * k;
                    const int uc = min(u, nu - 1);
                    const int x4 = (int)fdiv((uint32_t)uc, p.div_r2);
                    const int q = uc - x4 * NGRP * p.RHa;
                    const int hh = (int)fdiv((uint32_t)q, p.div_rha);
                    const int r = q - hh * p.RHa;
                    const int gy = g.yA + r * rstep;
                    const bool ok = u < nu && r < g.RH && gy >= 0 && gy < p.H;
                    x_hh[k] = u < nu ? hh : NGRP;
                    x_voff[k] = ok ? (uint32_t)(((hh * 8 * p.H + gy) * p.W + 4 * x4) * 2) : OOB;
#pragma unroll
                    for (int px = 0; px < 4; ++px)
                        x_lds[k][px] = (q * p.pitch + p.padl + 4 * x4 + px) * 16;
                }
            } else if constexpr (XD) {
                const int W2 = p.W >> 1;
                const int nu = NGRP * p.RHa * W2;
#pragma unroll
                for (int k = 0; k < XDM; ++k) {
                    const int u = mt + 256 * k;
                    const int uc = min(u, nu - 1);
                    const int x2 = (int)fdiv((uint32_t)uc, p.div_r2);
                    const int q = uc - x2 * NGRP * p.RHa;
                    const int hh = (int)fdiv((uint32_t)q, p.div_rha);
                    const int r = q - hh * p.RHa;
                    const int gy = g.yA + r * rstep;
                    const bool ok = u < nu && r < g.RH && gy >= 0 && gy < p.H;
                    x_hh[k] = u < nu ? hh : NGRP;
                    x_voff[k] = ok ? (uint32_t)(((hh * 8 * p.H + gy) * p.W + 2 * x2) * 2) : OOB;
#pragma unroll
                    for (int px = 0; px < 2; ++px)
                        x_lds[k][px] = (q * p.pitch + p.padl + 2 * x2 + px) * 16;
                }
            } else {
                const int nu = NGRP * p.RHa * p.W;
#pragma unroll
                for (int k = 0; k < XSM; ++k) {
                    const int u = mt + 256 * k;
                    const int uc = min(u, nu - 1);
                    const int q = (int)fdiv((uint32_t)uc, p.div_w);
                    const int xg = uc - q * p.W;
                    const int hh = (int)fdiv((uint32_t)q, p.div_rha);
                    const int r = q - hh * p.RHa;
                    const int gy = g.yA + r * rstep;
                    const bool ok = u < nu && r < g.RH && gy >= 0 && gy < p.H;
                    x_hh[k] = u < nu ? hh : NGRP;
                    x_voff[k] = ok ? (uint32_t)(((hh * 8 * p.H + gy) * p.W + xg) * 2) : OOB;
                    x_lds[k][0] = (q * p.pitch + p.padl + xg) * 16;
                }
            }
            if constexpr (!PACKED) {
#pragma unroll
                for (int k = 0; k < WU; ++k) {
                    // unit = (output channel, 8-channel group of the pass); group 2*gp + h belongs to
                    // lane half h of step block gp
                    const int u = mt + 256 * k;
                    const int col = u / NGRP, hh = u % NGRP;
                    const int co = g.cg * TN + col;
                    const bool ok = u < TN * NGRP && co < p.Cout;
                    w_hh[k] = u < TN * NGRP ? hh : NGRP;
                    w_voff[k] = ok ? (uint32_t)(((co * p.Cin + hh * 8) * T) * 2) : OOB;
                    w_lds[k] = ((((hh >> 1) * T * NCB + (col >> 5)) * 2 + (hh & 1)) * 32 + ((col & 31) ^ ((hh & 1) * 8))) * 16;
                }
            }
        };

        // request the input rows (and, unless packed, the weights) of pass ck into the registers
        auto request = [&](const Geom &g, int ck) __attribute__((always_inline)) {
            const int live = (p.Cin >> 3) - ck * NGRP;          // groups of this pass that exist (the rest: padding)
            // (the same for the whole wavefront: said explicitly, or the 2-byte loads below each get a
            // loop over the distinct values of a vector register)
            const uint32_t xbase = (uint32_t)__builtin_amdgcn_readfirstlane(
                (int)(((uint32_t)g.n * (uint32_t)p.Cin + (uint32_t)(ck * NGRP * 8)) * chbytes));
#pragma unroll
            for (int k = 0; k < NXU; ++k) {
                if (!XV && k >= p.xu) break;
                const uint32_t voff = x_hh[k] >= live ? OOB : x_voff[k];
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    if constexpr (XV) {
                        const uint32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rx, voff, xbase + c * chbytes, 0);
                        xv[k][c][0] = v.x; xv[k][c][1] = v.y; xv[k][c][2] = v.z; xv[k][c][3] = v.w;
                    } else if constexpr (XQ) {
                        const uint32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rx, voff, xbase + c * chbytes, 0);
                        xq[k][c][0] = v.x; xq[k][c][1] = v.y;
                    } else if constexpr (XD) {
                        xd[k][c] = __builtin_amdgcn_raw_buffer_load_b32(rx, voff, xbase + c * chbytes, 0);
                    } else {
                        xs[k][c] = __builtin_amdgcn_raw_buffer_load_b16(rx, voff, xbase + c * chbytes, 0);
                    }
                }
            }
            if constexpr (!PACKED) {
                const uint32_t wbase = (uint32_t)ck * (uint32_t)(NGRP * 8 * T * 2);
#pragma unroll
                for (int k = 0; k < WU; ++k) {
                    const uint32_t voff = w_hh[k] >= live ? OOB : w_voff[k];
#pragma unroll
                    for (int i = 0; i < T; ++i) {
                        const uint32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rw, voff + 16 * i, wbase, 0);
                        wr[k][4 * i + 0] = v.x; wr[k][4 * i + 1] = v.y; wr[k][4 * i + 2] = v.z; wr[k][4 * i + 3] = v.w;
                    }
                }
            }
        };

        // transpose the registers into pass buffer b
        auto commit = [&](int b) __attribute__((always_inline)) {
            uint8_t *xl = smem + b * p.lds_buf_bytes + p.lds_w_bytes;
#pragma unroll
            for (int k = 0; k < NXU; ++k) {
                if (!XV && k >= p.xu) break;
                if (x_hh[k] < NGRP) {
                    if constexpr (XV) {
#pragma unroll
                        for (int px = 0; px < 8; ++px) {
                            const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
                            uint32x4 d;
                            d.x = __builtin_amdgcn_perm(xv[k][1][px >> 1], xv[k][0][px >> 1], sel);
                            d.y = __builtin_amdgcn_perm(xv[k][3][px >> 1], xv[k][2][px >> 1], sel);
                            d.z = __builtin_amdgcn_perm(xv[k][5][px >> 1], xv[k][4][px >> 1], sel);
                            d.w = __builtin_amdgcn_perm(xv[k][7][px >> 1], xv[k][6][px >> 1], sel);
                            *reinterpret_cast<uint32x4 *>(xl + x_lds[k][px]) = d;
                        }
                    } else if constexpr (XQ) {
#pragma unroll
                        for (int px = 0; px < 4; ++px) {
                            const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
                            uint32x4 d;
                            d.x = __builtin_amdgcn_perm(xq[k][1][px >> 1], xq[k][0][px >> 1], sel);
                            d.y = __builtin_amdgcn_perm(xq[k][3][px >> 1], xq[k][2][px >> 1], sel);
                            d.z = __builtin_amdgcn_perm(xq[k][5][px >> 1], xq[k][4][px >> 1], sel);
                            d.w = __builtin_amdgcn_perm(xq[k][7][px >> 1], xq[k][6][px >> 1], sel);
                            *reinterpret_cast<uint32x4 *>(xl + x_lds[k][px]) = d;
                        }
                    } else if constexpr (XD) {
#pragma unroll
                        for (int px = 0; px < 2; ++px) {
                            const uint32_t sel = px ? 0x07060302u : 0x05040100u;
                            uint32x4 d;
                            d.x = __builtin_amdgcn_perm(xd[k][1], xd[k][0], sel);
                            d.y = __builtin_amdgcn_perm(xd[k][3], xd[k][2], sel);
                            d.z = __builtin_amdgcn_perm(xd[k][5], xd[k][4], sel);
                            d.w = __builtin_amdgcn_perm(xd[k][7], xd[k][6], sel);
                            *reinterpret_cast<uint32x4 *>(xl + x_lds[k][px]) = d;
                        }
                    } else {
                        // the eight loads of a unit stay eight registers until here: packed in pairs
                        // where they are requested, every pair would wait for its own memory round trip
#pragma unroll
                        for (int c = 0; c < 8; ++c) asm volatile("" : "+v"(xs[k][c]));
                        uint32x4 d;
                        d.x = (uint32_t)xs[k][0] | ((uint32_t)xs[k][1] << 16);
                        d.y = (uint32_t)xs[k][2] | ((uint32_t)xs[k][3] << 16);
                        d.z = (uint32_t)xs[k][4] | ((uint32_t)xs[k][5] << 16);
                        d.w = (uint32_t)xs[k][6] | ((uint32_t)xs[k][7] << 16);
                        *reinterpret_cast<uint32x4 *>(xl + x_lds[k][0]) = d;
                    }
                }
            }
            if constexpr (!PACKED) {
                uint8_t *wl = smem + b * p.lds_buf_bytes;
#pragma unroll
                for (int k = 0; k < WU; ++k) {
                    if (w_hh[k] < NGRP) {
#pragma unroll
                        for (int t = 0; t < T; ++t) {
                            uint32_t d[4];
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                // halves (channel 2q, tap t) and (channel 2q+1, tap t) of the unit's 8 x T block
                                const int e0 = (2 * q) * T + t, e1 = (2 * q + 1) * T + t;
                                const uint32_t sel =
                                    ((e0 & 1) ? 0x00000302u : 0x00000100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
                                d[q] = __builtin_amdgcn_perm(wr[k][e1 >> 1], wr[k][e0 >> 1], sel);
                            }
                            uint32x4 dv;
                            dv.x = d[0]; dv.y = d[1]; dv.z = d[2]; dv.w = d[3];
                            *reinterpret_cast<uint32x4 *>(wl + w_lds[k] + t * NCB * 64 * 16) = dv;
                        }
                    }
                }
            }
        };

        // packed weights of pass ck of channel block cg: global memory -> pass buffer b directly
        // (no registers; each wavefront instruction moves 64 consecutive fragments)
        auto weights_direct = [&](int cg, int ck, int b) __attribute__((always_inline)) {
            if constexpr (PACKED) {
                const uint32_t soff = (uint32_t)((cg * npass + ck) * WITEMS) * 16u;
                constexpr int ROUNDS = (WITEMS / 64 + 3) / 4;
#pragma unroll
                for (int k = 0; k < ROUNDS; ++k) {
                    const int i = mwave + 4 * k;                           // 64-fragment slice of the pass
                    if (i * 64 < WITEMS)
                        __builtin_amdgcn_raw_ptr_buffer_load_lds(
                            rw, (__attribute__((address_space(3))) void *)(smem + b * p.lds_buf_bytes + i * 1024), 16,
                            (i * 64 + lane) * 16, soff, 0, 0);
                }
            }
        };
        // ... and the wait for them: everything this wavefront has requested has arrived
        auto weights_landed = [&]() __attribute__((always_inline)) {
            if constexpr (PACKED) __builtin_amdgcn_s_waitcnt(0 | (0x7 << 4) | (0xF << 8));    // vmcnt(0)
        };

        // the padding columns of the staged rows, both buffers (the output staging overwrites them)
        auto zero_pads = [&]() __attribute__((always_inline)) {
            const int npad = p.pitch - p.W;
            const int per = NGRP * p.RHa * npad;
            for (int u = mt; u < 2 * per; u += 256) {
                const int b = u >= per ? 1 : 0;
                const int v = u - b * per;
                const int rowi = v / npad;
                const int c = v - rowi * npad;
                const int col = c < p.padl ? c : p.W + c;
                xbuf(b)[rowi * p.pitch + col] = make_uint4(0, 0, 0, 0);
            }
        };

        // Per period (the multiplying wavefronts are on pass ck of the item): write pass ck+1, whose
        // registers were requested a period ago, to the other buffer; start its packed weights;
        // request pass ck+2 (or pass 0 / 1 of the next item).  The registers are free again only
        // after the commit, so one pass is in flight at a time, for a whole period.
        Geom g = geom_at(item, 0);
        setup(g);
        request(g, 0);
        for (;;) {
            int item2 = item, ti2 = ti, ntile2 = ntile;
            const bool more = next_pos(item2, ti2, ntile2);
            const Geom gn = more ? geom_at(item2, ti2) : g;
            commit(0);
            weights_direct(g.cg, 0, 0);
            zero_pads();
            if (npass > 1) request(g, 1);
            weights_landed();                                  // (waits for the request too: once per item)
            __syncthreads();                                   // P
            for (int ck = 0; ck < npass; ++ck) {
                if (ck + 1 < npass) {
                    commit((ck + 1) & 1);
                    weights_direct(g.cg, ck + 1, (ck + 1) & 1);
                    if constexpr (XV) {
                        // the packed weights have the rest of the period to land: wait until only
                        // the request that follows them is still in flight
                        if (ck + 2 < npass) {
                            request(g, ck + 2);
                            if constexpr (PACKED) __builtin_amdgcn_s_waitcnt((8 * XU) | (0x7 << 4) | (0xF << 8));
                        } else {
                            weights_landed();
                        }
                    } else {
                        weights_landed();
                        if (ck + 2 < npass) request(g, ck + 2);
                    }
                }
                __syncthreads();                    // B_ck
            }
            // the next item's first pass flies under the result stores
            if (more) { setup(gn); request(gn, 0); }
            __syncthreads();                                   // E1
            if constexpr (POOL) pool_out(g);
            else store_out(g);
            __syncthreads();                                   // E2
            if (!more) break;
            g = gn; item = item2; ti = ti2; ntile = ntile2;
        }
        return;
    }

    // ---- the multiplying wavefronts ----
    const int wm = wave % WM, wn = wave / WM;
    for (bool more = true; more; more = next_pos(item, ti, ntile)) {
        const Geom g = geom_at(item, ti);
        constexpr int KW = T == 25 ? 5 : (T == 9 ? 3 : 1);   // the window is square: T = KW * KW taps
        int xc[PXB][KW];
#pragma unroll
        for (int pb = 0; pb < PXB; ++pb) {
            const int m = g.m0 + (wm * PXB + pb) * 32 + c32;
            const int mm = min(m, g.mend - 1);                 // (pixels past the tile's end: computed, never stored)
            const int oy = (int)fdiv((uint32_t)mm, p.div_ow);
            const int ox = mm - oy * p.OW;
            const int pbase = (h * p.RHa + (oy - g.oyA) * (p.row_skip ? 1 : p.sh)) * p.pitch;
            const int pcol = (p.padl - p.pw) + ox * p.sw;
#pragma unroll
            for (int kx = 0; kx < KW; ++kx) xc[pb][kx] = pbase + pcol + kx * p.dw;
        }
        floatx16 acc[CHB][PXB];
#pragma unroll
        for (int cb = 0; cb < CHB; ++cb)
#pragma unroll
            for (int pb = 0; pb < PXB; ++pb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;
        __syncthreads();                                       // P

        // Residual layer: the added tensor is read in the accumulators' own layout -- a lane's four
        // consecutive pixels of one channel are 8 bytes -- and requested before the last pass, so
        // the loads (64 cache lines per instruction: lanes are channels) land under its MFMAs.
        uint32_t rres[RES ? CHB : 1][RES ? PXB : 1][4][2];
        auto request_residual = [&]() __attribute__((always_inline)) {
            if constexpr (!RES) return;
            const __amdgpu_buffer_rsrc_t rr = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<uint16_t *>(res), 0, (int)((size_t)p.N * p.Cout * ohw * 2), 0x00020000);
            const bool vec = (ohw & 3) == 0;
#pragma unroll
            for (int cb = 0; cb < CHB; ++cb) {
                const int co = g.cg * TN + (wn * CHB + cb) * 32 + c32;
#pragma unroll
                for (int pb = 0; pb < PXB; ++pb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int m = g.m0 + (wm * PXB + pb) * 32 + 8 * q + 4 * h;
                        const uint32_t off = (uint32_t)((((size_t)g.n * p.Cout + co) * ohw + m) * 2);
                        if (vec) {
                            const uint32x2 v = __builtin_amdgcn_raw_buffer_load_b64(rr, (co < p.Cout && m < ohw) ? off : OOB, 0, 0);
                            rres[cb][pb][q][0] = v.x; rres[cb][pb][q][1] = v.y;
                        } else {
                            uint32_t e[4];
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                e[k] = __builtin_amdgcn_raw_buffer_load_b16(rr, (co < p.Cout && m + k < ohw) ? off + 2 * k : OOB, 0, 0);
                            rres[cb][pb][q][0] = e[0] | (e[1] << 16); rres[cb][pb][q][1] = e[2] | (e[3] << 16);
                        }
                    }
            }
        };
        for (int ck = 0; ck < npass; ++ck) {
            if constexpr (RES) { if (ck == npass - 1) request_residual(); }
            const uint4 *wl = wbuf(ck & 1) + (wn * CHB * 2 + h) * 32 + (c32 ^ (h * 8));
            const uint4 *xl = xbuf(ck & 1);
            const int rowstep = p.dh * p.pitch;
            Frag a[2][CHB], b[2][PXB];
            auto load = [&](int s, int slot) __attribute__((always_inline)) {
                const int gp = s / T, tap = s % T;               // step = (pair of channel groups, tap)
                const int ky = tap / KW, kx = tap % KW;
                const int xgrp = gp * 2 * p.RHa * p.pitch;
#pragma unroll
                for (int cb = 0; cb < CHB; ++cb) a[slot][cb].u = wl[(s * NCB + cb) * 64];
#pragma unroll
                for (int pb = 0; pb < PXB; ++pb) b[slot][pb].u = xl[xc[pb][kx] + ky * rowstep + xgrp];
            };
            // the reads of step s+1 are issued before the MFMAs of step s and stay there (left to
            // itself the scheduler sinks them to their first use, and the matrix core idles for
            // an LDS round trip per step)
            load(0, 0);
#pragma unroll
            for (int s = 0; s < NG * T; ++s) {
                if (s + 1 < NG * T) load(s + 1, (s + 1) & 1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int cb = 0; cb < CHB; ++cb)
#pragma unroll
                    for (int pb = 0; pb < PXB; ++pb)
                        acc[cb][pb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[s & 1][pb].h, a[s & 1][cb].h,
                                                                             acc[cb][pb], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            __syncthreads();                                   // B_ck
        }

        // accumulators -> LDS [channel][pixel].  Accumulator register r of lane l is output
        // channel l%32 of its block, pixel 8*(r/4) + 4*(l/32) + r%4: four consecutive registers
        // are four consecutive pixels.  OP = TM/2 + 2 dwords per channel spreads the 32 channels
        // of a write over all banks.
        {
            const half2v z = {(_Float16)0.0f, (_Float16)0.0f};
#pragma unroll
            for (int cb = 0; cb < CHB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PXB; ++pb)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        if constexpr (RES) {     // added to the fp32 sums: one rounding
                            const half2v r0 = __builtin_bit_cast(half2v, rres[cb][pb][q][0]);
                            const half2v r1 = __builtin_bit_cast(half2v, rres[cb][pb][q][1]);
                            acc[cb][pb][4 * q] += (float)r0.x;     acc[cb][pb][4 * q + 1] += (float)r0.y;
                            acc[cb][pb][4 * q + 2] += (float)r1.x; acc[cb][pb][4 * q + 3] += (float)r1.y;
                        }
                        half2v v0, v1;
                        v0.x = (_Float16)acc[cb][pb][4 * q];     v0.y = (_Float16)acc[cb][pb][4 * q + 1];
                        v1.x = (_Float16)acc[cb][pb][4 * q + 2]; v1.y = (_Float16)acc[cb][pb][4 * q + 3];
                        if (p.relu) {            // clipping the rounded value = rounding the clipped value
                            v0 = __builtin_elementwise_max(v0, z);
                            v1 = __builtin_elementwise_max(v1, z);
                        }
                        uint2 v;
                        v.x = __builtin_bit_cast(uint32_t, v0);
                        v.y = __builtin_bit_cast(uint32_t, v1);
                        const int ch = (wn * CHB + cb) * 32 + c32;
                        *reinterpret_cast<uint2 *>(outl + ch * OP + (wm * PXB + pb) * 16 + 4 * q + 2 * h) = v;
                    }
        }
        __syncthreads();                                       // E1
        if constexpr (POOL) pool_out(g);
        else store_out(g);
        __syncthreads();                                       // E2
    }
}

// Rewrites w[Cout][Cin][kh][kw] into the order the passes of merit_conv2d_chws read it: for every
// channel block and pass the T * NCB * 64 fragments of 8 input channels in their LDS places.
// One thread per 16-byte fragment.
__global__ __launch_bounds__(256) void merit_conv2d_pack_w(ConvParams p, int T, int NCB, int NG, const uint16_t *__restrict__ w,
                                                          uint4 *__restrict__ out, long long total)
{
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int witems = NG * T * NCB * 64;
    const long long blk = i / witems;                      // (channel block, pass)
    int r = (int)(i - blk * witems);
    const int cg = (int)(blk / p.nchunks), ck = (int)(blk - (long long)cg * p.nchunks);
    const int s = r / (NCB * 64);                          // step = (pair of channel groups, tap)
    r -= s * NCB * 64;
    const int gp = s / T, t = s - gp * T;
    const int cb = r >> 6, hh = (r >> 5) & 1, slot = r & 31;
    const int cc = slot ^ (hh * 8);
    const int co = (cg * NCB + cb) * 32 + cc;
    const int ci0 = ((ck * NG + gp) * 2 + hh) * 8;
    uint32_t d[4] = {0, 0, 0, 0};
    if (co < p.Cout) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
            if (ci0 + c < p.Cin)
                d[c >> 1] |= (uint32_t)w[((size_t)co * p.Cin + ci0 + c) * T + t] << (16 * (c & 1));
    }
    out[i] = make_uint4(d[0], d[1], d[2], d[3]);
}

namespace {

template <typename K>
hipError_t launch_one(K kernel, const ConvParams &p, const void *x, const void *w, const void *res, void *y, hipStream_t s,
                      uint32_t grid)
{
    // raise this instance's dynamic-LDS limit to the 160 KB a gfx950 workgroup may use, once
    static std::atomic<int> raised{0};
    if (hipError_t e = raise_lds_limit_once(reinterpret_cast<const void *>(kernel), raised); e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(grid), dim3((unsigned)(p.NW * 64)), (size_t)p.lds_total, s, p, reinterpret_cast<const uint16_t *>(x),
                       reinterpret_cast<const uint16_t *>(w), reinterpret_cast<const uint16_t *>(res),
                       reinterpret_cast<uint16_t *>(y));
    return hipGetLastError();
}

template <int PXB, int CHB, int WM, int WN, int NG = 1, bool POOLS = false>
hipError_t launch_tile(const ConvParams &p, const void *x, const void *w, const void *res, void *y, hipStream_t s,
                       uint32_t grid, bool packed)
{
    // 8-pixel units per moving thread (1, 2); 4: four-pixel units (W % 4 == 0, 3x3 and 1x1 windows); 3: two-pixel units
    // (W % 4 == 2, the same windows, no added tensor, no pooling); 0: one-pixel units
    const int xu = (p.W & 7) == 0 ? p.xu : (p.xq == 1 ? 4 : (p.xq == 2 ? 3 : 0));
    const int T = p.kh * p.kw;
    if (p.residual) {
        // residual layer: 3x3 and 1x1 windows on the caller's weights, the two 64-channel tilings (on the
        // others the 32 registers of the added tensor would spill)
        if constexpr (POOLS && WN == 1) {
            if ((T != 9 && T != 1) || packed || p.pool) return hipErrorInvalidValue;
            if (T == 1) {
                if (xu == 1) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 1, 1, false, NG, false, true>, p, x, w, res, y, s, grid);
                if (xu == 2) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 1, 2, false, NG, false, true>, p, x, w, res, y, s, grid);
                if (xu == 4) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 1, 4, false, NG, false, true>, p, x, w, res, y, s, grid);
                return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 1, 0, false, NG, false, true>, p, x, w, res, y, s, grid);
            }
            if constexpr (NG != 4) {        // (64 channels per pass: 1x1 windows only)
                if (xu == 1) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 1, false, NG, false, true>, p, x, w, res, y, s, grid);
                if (xu == 2) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 2, false, NG, false, true>, p, x, w, res, y, s, grid);
                if (xu == 4) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 4, false, NG, false, true>, p, x, w, res, y, s, grid);
                return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 0, false, NG, false, true>, p, x, w, res, y, s, grid);
            }
        }
        return hipErrorInvalidValue;
    }
    if (p.pool) {
        // fused pooling: 3x3 windows on the caller's weights; not the 128-channel tiling on 8 wavefronts
        if constexpr (POOLS && NG != 4) {
            if (T != 9 || packed) return hipErrorInvalidValue;
            if (xu == 1) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 1, false, NG, true>, p, x, w, res, y, s, grid);
            if (xu == 2) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 2, false, NG, true>, p, x, w, res, y, s, grid);
            if (xu == 4) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 4, false, NG, true>, p, x, w, res, y, s, grid);
            return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, 9, 0, false, NG, true>, p, x, w, res, y, s, grid);
        }
        return hipErrorInvalidValue;
    }
#define MERIT_CHWS(Tv, XUv)                                                                             \
    do {                                                                                                \
        if (packed) return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, Tv, XUv, true, NG>, p, x, w, res, y, s, grid);  \
        return launch_one(merit_conv2d_chws<PXB, CHB, WM, WN, Tv, XUv, false, NG>, p, x, w, res, y, s, grid);    \
    } while (0)
    if constexpr (NG != 4) {
        if (T == 9 && xu == 1) MERIT_CHWS(9, 1);
        if (T == 9 && xu == 2) MERIT_CHWS(9, 2);
        if (T == 9 && xu == 0) MERIT_CHWS(9, 0);
        if (T == 9 && xu == 4) MERIT_CHWS(9, 4);
        if (T == 9 && xu == 3) MERIT_CHWS(9, 3);
    }
    if (T == 1 && xu == 1) MERIT_CHWS(1, 1);
    if (T == 1 && xu == 2) MERIT_CHWS(1, 2);
    if (T == 1 && xu == 0) MERIT_CHWS(1, 0);
    if (T == 1 && xu == 4) MERIT_CHWS(1, 4);
    if (T == 1 && xu == 3) MERIT_CHWS(1, 3);
    // 5x5 windows: the 256-pixel x 64-channel tiling only (a pass's 25 x 2 x 64 weight fragments are 51 KB)
    if constexpr (PXB == 2 && CHB == 2 && WM == 4 && WN == 1 && NG == 1) {
        if (T == 25 && xu == 1) MERIT_CHWS(25, 1);
        if (T == 25 && xu == 2) MERIT_CHWS(25, 2);
        if (T == 25 && xu == 0) MERIT_CHWS(25, 0);
    }
#undef MERIT_CHWS
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_conv2d_chws(const ConvParams &p, const void *x, const void *w, const void *res, void *y, hipStream_t s,
                              bool packed)
{
    if ((p.residual != 0) != (res != nullptr)) return hipErrorInvalidValue;
    const int64_t nitems = p.pool ? (int64_t)p.N * p.NB * p.co_groups : (int64_t)p.N * p.tiles_per_image * p.co_groups;
    if (nitems == 0) return hipSuccess;
    const int64_t slots = device_cu_count();            // one 512-thread workgroup per compute unit
    const uint32_t grid = (uint32_t)(nitems < slots ? nitems : slots);
    if (p.nchi == 8) {
        // 1x1 windows on 128 and more channels: 64 channels per pass on every tiling (a pass of 16 or 32
        // channels x one tap is a few MFMAs per wavefront: shorter than the barrier and the memory round trip)
        if (p.CB == 4 && p.NW == 12) return launch_tile<2, 2, 4, 2, 4, false>(p, x, w, res, y, s, grid, packed);
        if (p.CB == 4) return launch_tile<4, 2, 2, 2, 4, false>(p, x, w, res, y, s, grid, packed);
        if (p.TM == 128 && p.CB == 1) return launch_tile<1, 1, 4, 1, 4, false>(p, x, w, res, y, s, grid, packed);
        if (p.TM == 128) return launch_tile<1, 2, 4, 1, 4, true>(p, x, w, res, y, s, grid, packed);
        return launch_tile<2, 2, 4, 1, 4, true>(p, x, w, res, y, s, grid, packed);
    }
    if (p.CB == 4 && p.NW == 12) return launch_tile<2, 2, 4, 2, 1, true>(p, x, w, res, y, s, grid, packed);   // 256 x 128, 8 x (64 x 64)
    if (p.CB == 4) return launch_tile<4, 2, 2, 2>(p, x, w, res, y, s, grid, packed);     // 256 pixels x 128 channels, 4 x (128 x 64)
    if (p.TM == 128 && p.CB == 1) return launch_tile<1, 1, 4, 1, 2, false>(p, x, w, res, y, s, grid, packed);   // 128 pixels x 32 channels, 4 x (32 x 32)
    if (p.TM == 128) return launch_tile<1, 2, 4, 1, 2, true>(p, x, w, res, y, s, grid, packed);   // 128 pixels x 64 channels, 4 x (32 x 64), 32 channels per pass
    return launch_tile<2, 2, 4, 1, 1, true>(p, x, w, res, y, s, grid, packed);           // 256 pixels x 64 channels, 4 x (64 x 64)
}

hipError_t launch_conv2d_pack_weights(const ConvParams &p, const void *w, void *packed, hipStream_t s)
{
    const int T = p.kh * p.kw;
    const int NG = p.nchi / 2;
    const long long total = (long long)p.co_groups * p.nchunks * NG * T * p.CB * 64;
    if (total == 0) return hipSuccess;
    hipLaunchKernelGGL(merit_conv2d_pack_w, dim3((uint32_t)((total + 255) / 256)), dim3(256), 0, s, p, T, p.CB, NG,
                       reinterpret_cast<const uint16_t *>(w), reinterpret_cast<uint4 *>(packed), total);
    return hipGetLastError();
}

// ---- the packed copy in a buffer of the library's own, for callers that cannot allocate ----
// A file-scope device array: every GPU the library runs on holds its own copy at its own
// address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returned, per device.
static __device__ __align__(256) unsigned char scratch[MERIT_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void *scratch_ptr[MAX_DEVICES];          // device address of `scratch` on each GPU, once asked for

hipError_t scratch_address(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));      // the current device's copy
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_ptr[dev] = ptr;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

hipError_t launch_conv2d_chws_noalloc(const ConvParams &p, const void *x, const void *w, void *y, hipStream_t s)
{
    void *packed = nullptr;
    hipError_t e = scratch_address(&packed);
    if (e != hipSuccess) return e;
    e = launch_conv2d_pack_weights(p, w, packed, s);            // writes every fragment the passes read
    if (e != hipSuccess) return e;
    return launch_conv2d_chws(p, x, packed, nullptr, y, s, true);
}

}  // namespace merit
