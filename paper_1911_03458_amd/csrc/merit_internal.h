// Internal declarations shared by the host plan code and the HIP kernels.
// Not part of the public ABI (that is include/merit.h).
#pragma once

#include <stdint.h>
#include <atomic>
#include <hip/hip_runtime.h>

#include "merit.h"

namespace merit {

// ---- small integer helpers -------------------------------------------------

// q = n / d as (n * magic) >> 32 with magic = floor(2^32 / d) + 1.  Exact for
// every n with (n + d) * d < 2^32; the plan code checks that bound for each use.
struct FastDiv {
    uint32_t d;
    uint32_t magic;
};
inline FastDiv make_fastdiv(uint32_t d)
{
    FastDiv f;
    f.d = d;
    f.magic = d == 1u ? 0u : (uint32_t)((0x100000000ull / d) + 1ull);   // d == 1 does not fit: see fdiv
    return f;
}
#ifdef __HIPCC__
__device__ __forceinline__ uint32_t fdiv(uint32_t n, FastDiv f)
{
    // d == 1 has magic 0 and adds n instead: a select, no branch
    return __umulhi(n, f.magic) + (f.d == 1u ? n : 0u);
}

// Consecutive hardware workgroup ids go to the 8 XCDs in turn, each with an L2 of its own.
// With xq = grid / 8 and xr = grid % 8, XCD x gets the x-th contiguous run of the work list
// (a band of image rows for row-major lists), so its L2 fetches that band and its halo once
// instead of a share of every row.  A bijection of [0, grid) for any grid.
__device__ __forceinline__ uint32_t xcd_band_item(uint32_t hw_id, int xq, int xr)
{
    const uint32_t xcd = hw_id & 7u, slot = hw_id >> 3;
    return xcd * (uint32_t)xq + min(xcd, (uint32_t)xr) + slot;
}

// Results of a convolution tile, LDS staging -> global, where a channel's run of the tile starts on
// any element of the output (OH*OW % 8 != 0; y itself is 16-byte aligned).  outl: [channel][TM / 2 + 2]
// dwords, two pixels each; a0: element index in y of channel 0's first pixel, channel c `ohw` elements
// further; cnt: pixels of the run (<= TM); nch: channels; t: thread of NT.  The 16-byte store units lie
// on the output's own 16-byte grid (one more per channel than the tile has, as the run may straddle):
// a unit that starts at tile pixel 0 <= px0 < own is five dwords of the staging row, shifted down by a
// half where px0 is odd (own <= cnt - 7: every stored unit is whole).  The up to 7 pixels before the
// first unit (`heads`) and behind the last (`tails`) go out as 2-byte stores in a pass of their own, 16
// lanes per channel (in one loop every wavefront would take both branches).  Tiles that abut pass
// own = cnt - 7 and both flags; tiles that overlap by 8 pixels pass own = TM - 8 and no flag, but for a
// plane's first tile (heads) and last tile (own = cnt - 7, tails).
template <int TM, int NT>
__device__ __forceinline__ void store_runs_on_grid(const uint32_t *outl, uint16_t *__restrict__ y, size_t a0, int ohw,
                                                   int cnt, int nch, int own, bool heads, bool tails, int t)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int OP = TM / 2 + 2, UPC = TM / 8 + 1;
    // (the LDS reads of two units per thread go out together, clamped to the area where a unit
    // is not stored: half the round trips, and few enough registers)
    constexpr int UB = 2;
#pragma unroll 1
    for (int u0 = t; u0 < nch * UPC; u0 += NT * UB) {
        uint32_t d[UB][5];
        int pxs[UB];
        uint32_t coff[UB];                                   // c * ohw (below 2^32: a tile's channels)
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            const int u = u0 + NT * i;
            const int c = min(u / UPC, nch - 1);
            const int j = u - (u / UPC) * UPC;
            coff[i] = (uint32_t)c * (uint32_t)ohw;
            const int px0 = 8 * j - (int)((a0 + coff[i]) & 7);   // tile pixel of the unit's first element
            pxs[i] = (u < nch * UPC && px0 >= 0 && px0 < own) ? px0 : -1;
            const uint32_t *src = outl + c * OP + (max(pxs[i], 0) >> 1);   // (the fifth dword: at most the row's padding)
#pragma unroll
            for (int q = 0; q < 5; ++q) d[i][q] = src[q];
        }
#pragma unroll
        for (int i = 0; i < UB; ++i) {
            if (pxs[i] < 0) continue;
            const uint32_t sh = (uint32_t)(pxs[i] & 1) * 16u;
            u32x4 v;
            v.x = __builtin_amdgcn_alignbit(d[i][1], d[i][0], sh);
            v.y = __builtin_amdgcn_alignbit(d[i][2], d[i][1], sh);
            v.z = __builtin_amdgcn_alignbit(d[i][3], d[i][2], sh);
            v.w = __builtin_amdgcn_alignbit(d[i][4], d[i][3], sh);
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4 *>(y + a0 + coff[i] + pxs[i]));
        }
    }
    if (!heads && !tails) return;
    constexpr int EB = 2;
#pragma unroll 1
    for (int e0 = t; e0 < nch * 16; e0 += NT * EB) {
        uint16_t ev[EB];
        int epx[EB];
        uint32_t eoff[EB];
#pragma unroll
        for (int i = 0; i < EB; ++i) {
            const int e = e0 + NT * i;
            const int c = min(e >> 4, nch - 1), k = e & 7;
            eoff[i] = (uint32_t)c * (uint32_t)ohw;
            const int head = min(cnt, (8 - (int)((a0 + eoff[i]) & 7)) & 7);
            const int px = (e & 8) ? (tails ? head + ((cnt - head) & ~7) + k : cnt) : ((heads && k < head) ? k : cnt);
            epx[i] = (e < nch * 16 && px < cnt) ? px : -1;
            ev[i] = reinterpret_cast<const uint16_t *>(outl + c * OP)[max(epx[i], 0)];
        }
#pragma unroll
        for (int i = 0; i < EB; ++i)
            if (epx[i] >= 0) y[a0 + eoff[i] + epx[i]] = ev[i];
    }
}
#endif

// ---- launcher helpers (host) -------------------------------------------------
// A kernel instance may use more than 64 KB of dynamic LDS only after its limit has been raised
// (to the 160 KB a gfx950 workgroup may use).  Once per instance; `done` is the instance's
// flag (a function-local static of the launcher template).  Safe to call from several threads:
// the attribute call is idempotent, the flag only saves repeating it.
inline hipError_t raise_lds_limit_once(const void *kernel, std::atomic<int> &done)
{
    if (!done.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        done.store(1, std::memory_order_release);
    }
    return hipSuccess;
}
int device_cu_count();          // compute units of the current device (256 on MI355X); cached, thread-safe

// ---- pooling ---------------------------------------------------------------
enum PoolVariant { POOL_TILE_GENERIC = 0, POOL_ROWS_K3S2P1 = 1, POOL_ROWS_K2S2P0 = 2, POOL_ROWS_K3S1P1 = 3,
                   POOL_STREAM_K3S2P1 = 4, POOL_PLANE = 5, POOL_LANES_K3S2 = 6, POOL_LANES2_K3S2 = 7 };

struct PoolParams {
    int NC, H, W, OH, OW;
    int kh, kw, sh, sw, ph, pw;
    int is_avg;
    int variant;
    int TH, TW;            // outputs per workgroup tile
    int tiles_y, tiles_x;
    int RH, RW, pitch;     // staged region (rows, cols) and LDS row pitch in floats
    FastDiv div_tiles_x, div_tiles_y;
    FastDiv div_rw;        // generic: staged columns
    FastDiv div_tw;        // generic: tile columns
    FastDiv div_p4;        // rows variant: float4 per staged row
    FastDiv div_ow4;       // rows variant: float4 per output row
    int lg_shift;          // stream variant: log2(lanes per (plane, strip) item)
    int items;             // stream variant: NC * strips
    int grid;              // workgroups to launch
};

// ---- block matching --------------------------------------------------------
enum SadVariant { SAD_GENERIC = 0, SAD_ROWSCAN_B16 = 1, SAD_ROWSCAN_PAIR = 2 };

struct SadParams {
    int H, W, B, R, n;     // n = 2R+1 candidates per axis
    int nby, nbx;
    int win;               // B + 2R: search window edge in pixels
    int pitch;             // LDS bytes per window row (multiple of 4)
    int variant;
    int bpw;               // blocks per workgroup (rowscan variant)
    int groups_x;          // workgroups per block row (rowscan variant)
    int xq, xr;            // grid / 8, grid % 8 (see xcd_band_item)
    FastDiv div_n;
    FastDiv div_win4;      // dwords per staged window row
    FastDiv div_nbx;
};

// ---- convolution -----------------------------------------------------------
enum ConvVariant { CONV_PLANAR_SMALLC = 0, CONV_CHBLOCK = 1, CONV_DIRECT = 2, CONV_CHWS = 3 };

struct ConvParams {
    int N, Cin, H, W, Cout, OH, OW;
    int kh, kw, sh, sw, ph, pw;
    int dh, dw;            // input rows / columns per step of the window indices (dilation)
    int variant;
    int TM;                // output pixels (linear, row-major within an image) per workgroup
    int PXW;               // 32-pixel blocks per wave
    int NW;                // wavefronts per workgroup (4 or 8)
    int CB;                // 32-channel output blocks per workgroup
    int tiles_per_image;
    int co_groups;         // grid.y
    int rows_out_max;      // output rows a tile can touch
    int RHa;               // staged input rows (allocated)
    int pitch;             // staged row pitch: halves (planar) or pixels (channel-blocked)
    int padl;              // staged column of input x = 0
    int G, G2;             // planar: (ci,ky) groups and padded-even count
    int S;                 // MFMA K-steps (K = 16 each)
    int nchi;              // channel-blocked: 8-channel groups per pass incl. zero padding (even)
    int nchunks;           // channel-blocked: passes over the channels (1: everything is staged at once)
    int lds_w_bytes;       // weights region
    int lds_x_bytes;       // input region
    int lds_o_offset;      // output staging region: byte offset and size
    int lds_o_bytes;
    int lds_total;         // LDS per workgroup
    int front;             // planar: slot of tap kx = 0 inside an 8-slot fragment (0 or 1)
    int aligned;           // planar: every fragment starts on an even staged column
    int relu;              // product function max(v1.v2, 0): results clipped at zero before rounding
    int residual;          // a tensor of the output's shape is added to the sums before clip and rounding
    int ws;                // planar: wave-specialised kernel (4 multiplier + 4 mover wavefronts)
    int su;                // wave-specialised kernel: unrolled K steps (S <= su <= S+2)
    int lg_chunks;         // wave-specialised kernel: log2 of the 16-byte chunks per staged row, rounded up
    int wg_per_cu;         // resident workgroups per compute unit the launcher sizes the grid for
    // convolution followed by 3x3 / stride 2 / padding 1 max pooling, fused (wave-specialised kernel only)
    int pool;              // 1: the workgroup pools its results in LDS and writes the pooled tensor
    int PH, PW;            // pooled output extent (OH/2, OW/2)
    int PB, NB;            // pooled rows per workgroup (band), bands per image
    int pw8;               // 8-pixel units per pooled row (PW/8)
    FastDiv div_ow;
    FastDiv div_kh;
    FastDiv div_pitch8;    // planar staging: 16-byte units per staged row
    FastDiv div_rha;
    FastDiv div_g2;
    FastDiv div_w8;        // channel-blocked staging: 8-pixel chunks per row
    FastDiv div_nchi;      // channel-blocked staging: channel groups per output channel
    FastDiv div_tiles;
    FastDiv div_nb;        // fused pooling: bands per image
    FastDiv div_pw8;       // fused pooling: units per pooled row
    // (ConvParams + the four pointers end in the sixth 64-byte kernel-argument line, where the grid
    // extents HIP appends follow: touch_kernarg_lines in conv2d.hip covers all six)
    int pipe;              // multi-pass kernel: 9 or 1 = taps of the pipelined vector staging, 0 = plain staging
    FastDiv div_w;         // multi-pass kernel, one-pixel staging units: W
    // wave-specialised multi-pass kernel (CONV_CHWS): CB = 32-channel blocks per workgroup (4 or 2),
    // TM = 256, nchi = 2 channel groups per pass, nchunks = passes
    int lds_buf_bytes;     // one of its two pass buffers (weights, then input rows)
    int xu;                // input staging units per moving thread and pass
    FastDiv div_cog;       // work item -> (tile, channel block)
    FastDiv div_r2;        // staged rows of both channel groups of a pass (2 * RHa)
    int pool_halo;         // fused pooling there: 1 = a tile computes the row above its first pooled row itself
    int xq;                // multi-pass kernel: the input rows are staged in units of 8 channels x 4 pixels (1) or x 2 pixels (2)
    int unal;              // wave-specialised few-channel kernel: 1 = image rows or output planes start on any element (W % 8 != 0 or OH*OW % 8 != 0)
    int row_skip;          // multi-pass kernel, windows one row high with a row stride: 1 = only the image rows that are used are staged
    int tile_px;           // output pixels from one tile's start to the next: TM; multi-pass kernel with whole-row tiles: rows * OW <= TM;
                           // wave-specialised few-channel kernel on output planes off the 16-byte grid: TM - 8 (tiles overlap by 8 pixels)
                           // (rows_out_max odd), 0 = that row is carried from the tile before it (rows_out_max even)
};

// ---- launchers (defined in the .hip files) --------------------------------
hipError_t launch_pool2d(const PoolParams &p, const float *x, float *y, hipStream_t s);
hipError_t launch_sad(const SadParams &p, const uint8_t *cur, const uint8_t *ref,
                      int32_t *sad, int32_t *mv, hipStream_t s);
hipError_t launch_conv2d(const ConvParams &p, const void *x, const void *w, const void *r, void *y, hipStream_t s);

const char *pool_kernel_name(const PoolParams &p);
const char *sad_kernel_name(const SadParams &p);
const char *conv_kernel_name(const ConvParams &p);
// wave-specialised multi-pass kernel: w is the [Cout][Cin][kh][kw] tensor, or (packed) what
// launch_conv2d_pack_weights wrote
hipError_t launch_conv2d_chws(const ConvParams &p, const void *x, const void *w, const void *res, void *y, hipStream_t s,
                              bool packed);
hipError_t launch_conv2d_pack_weights(const ConvParams &p, const void *w, void *packed, hipStream_t s);
// 3x3 / stride 2 / padding 1 max pooling of a binary16 tensor [planes][OH][OW] (OH, OW even): the
// second pass of a convolution + pooling plan that runs as two launches (csrc/maxpool_f16.hip)
hipError_t launch_maxpool_f16(const void *c, void *y, int64_t planes, int OH, int OW, hipStream_t s);
// the same two launches with the packed copy in the library's own fixed device buffer
// (MERIT_NOALLOC_SCRATCH_BYTES; the caller has checked that the plan's packed weights fit)
hipError_t launch_conv2d_chws_noalloc(const ConvParams &p, const void *x, const void *w, void *y, hipStream_t s);

// ---- correlation layer -----------------------------------------------------
// One staging unit = 8 pixels x 8 channels.  One unit per thread and pass measured best: fewer
// registers (five wavefronts per SIMD) beat fewer, larger passes.
constexpr int CORR_XB = 1;            // staging units a thread holds in registers per pass
constexpr int CORR_LDS_KB = 40;       // LDS per workgroup at most: four workgroups and more per CU
struct CorrParams {
    int N, C, H, W, R, sd, n;   // n = 2R+1 displacements per axis, sd = displacement stride
    int nchi;                   // channel groups of 8 (C padded)
    int chg;                    // channel groups staged per pass (a multiple of 4 = one MFMA reduction step)
    int xchunks;                // 64-pixel chunks per image row
    int cols2;                  // staged columns of the second tensor per chunk (multiple of 8)
    int lead;                   // columns staged left of the chunk's first pixel (multiple of 8, >= R*sd)
    int xq, xr;                 // grid / 8 and grid % 8: hardware workgroup id -> one contiguous band of work per XCD
    // staged rows are stored by residue class of the column modulo sd: position = class * pitch + column / sd
    int pitch1, P1;             // first tensor: positions per class (ceil(64/sd)), positions per channel group
    int pitch2, P2;             // second tensor: ceil(cols2/sd), sd * pitch2
    int nsb, nblk;              // 16-pixel blocks per class, blocks per chunk (sd * nsb <= 8)
    int nb;                     // 16-column blocks of the second tensor per pixel block: ceil((16 + 2R) / 16)
    FastDiv div_n, div_xchunks, div_h, div_sd;
    FastDiv div_perg, div_perg_last;   // staging units per channel group: full chunks, the last chunk of a row
};

// ---- depthwise convolution -----------------------------------------------------
enum DwVariant { DW_TILE_GENERIC = 0, DW_ROWS_K3S1P1 = 1 };

struct DwParams {
    int NC, C, H, W, OH, OW;
    int kh, kw, sh, sw, ph, pw;
    int variant;
    int TH, tiles_y;       // output rows per workgroup, workgroups per plane
    int pitch;             // generic: staged halves per row (W + 2*pw); rows variant: 16-byte chunks per row
    int lds_w_offset;      // generic: byte offset of the float weights
    int lds_bytes;
    FastDiv div_tiles_y, div_c, div_pitch;
    FastDiv div_ow;        // generic: OW; rows variant: W/8
};

hipError_t launch_dwconv(const DwParams &p, const void *x, const void *w, void *y, hipStream_t s);
const char *dwconv_kernel_name(const DwParams &p);

// ---- separable filter --------------------------------------------------------------
struct SepParams {
    int N, H, W, k;
    int c;                 // window offset: tap a reads coordinate p + a - c, c = k/2
    int c4;                // c rounded up to 4: the staged columns start at x0 - c4
    int TH;                // output rows per workgroup (a multiple of 4); 64 columns
    int tiles_y, tiles_x;
    int PI, PM;            // LDS row pitch (floats) of the staged input and of the row-pass result
    int lds_bytes;
    int wg_per_cu;         // persistent workgroups per compute unit
    FastDiv div_tiles_x, div_tiles_y, div_rh;
};

hipError_t launch_sepfilter(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                            hipStream_t s);

// ---- bilateral filter ----------------------------------------------------------------
struct BilatParams {
    int N, H, W, k;
    int c, c4;             // window offset k/2; the staged columns start at x0 - c4 (c rounded up to 4)
    int tiles_y, tiles_x;  // 16 x 64 output tiles
    int PI;                // LDS row pitch in floats (a multiple of 4)
    int lds_bytes;
    float scale;           // sqrt(|norm| log2 e): exp(d*d*norm) = 2^(-+ (d*scale)^2); set per call
    int neg;               // norm <= 0; set per call
    FastDiv div_tiles_x, div_tiles_y, div_p4;
};

hipError_t launch_bilateral(const BilatParams &p, const float *x, const float *gx, const float *gy, float *y,
                            hipStream_t s);

hipError_t launch_correlation(const CorrParams &p, const void *x1, const void *x2, void *y, hipStream_t s);
size_t corr_lds_bytes(const CorrParams &p);
int conv_direct_channels();     // output channels per workgroup of the one-element-per-thread convolution

}  // namespace merit

// ---- any descriptor: the definition, one thread per row ------------------------
namespace merit {
struct GenericOperand {
    int ndim;
    int shape[MERIT_MAX_DIMS];
    long long pitch[MERIT_MAX_DIMS];      // elements between neighbours along each axis (dense, row-major)
    int axis[MERIT_MAX_INDEX];            // d_j, -1: the index does not move this operand
    int stride[MERIT_MAX_INDEX];          // s_j
    int offset[MERIT_MAX_INDEX];          // o_j
};
struct GenericParams {
    int mode;                             // 0 dot product (binary16), 1 maximum, 2 mean (fp32)
    int pad;                              // merit_pad
    int relu;
    int n_par, n_acc;
    int range[MERIT_MAX_INDEX];
    long long rows;                       // product of the parallel ranges = output elements
    long long acc;                        // product of the accumulation ranges
    GenericOperand a, b;
};
hipError_t launch_generic(const GenericParams &p, const void *a, const void *b, void *y, hipStream_t s);
const char *generic_kernel_name(const GenericParams &p);
}  // namespace merit

struct merit_plan {
    merit_plan_desc desc;
    int64_t tile_req[MERIT_MAX_INDEX];   // caller's tile override, 0 = library default
    int32_t out_ndim;
    int64_t out_shape[MERIT_MAX_DIMS];
    merit::PoolParams pool;
    merit::SadParams sad;
    merit::ConvParams conv;
    merit::CorrParams corr;
    merit::DwParams dw;
    merit::SepParams sep;
    merit::BilatParams bil;
    int generic;                          // 1: no specialised kernel took the descriptor; `gen` runs it
    merit::GenericParams gen;
    merit_launch_info info;
    // convolution plans on the wave-specialised multi-pass kernel: the planner's estimate for the
    // chosen tiling, in units of one 256-pixel x 64-channel tile
    double est_units;
    // convolution + pooling plans that run as two launches (the plain convolution into a
    // stream-ordered temporary, then the binary16 pooling kernel): `conv2` is the plain convolution
    int two_pass;
    merit::ConvParams conv2;
};
