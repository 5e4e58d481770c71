// 2-D convolution for gfx950 as an implicit GEMM on the matrix cores.
//
// k = (n, co, oy, ox | ci, ky, kx)                        (Section III-C, Eq. 6)
//     M(x)[p,a] = x[n, ci, oy*sh + ky - ph, ox*sw + kx - pw]   (zero outside)
//     M(w)[p,a] = w[co, ci, ky, kx]
// reduced with the dot product (Section III-B, Eq. 3).  M(x) (the unrolled
// matrix U(A) of Section III-A) is never materialised: a workgroup stages the
// minimal covering sub-tensor of its pixel tile (Section IV-A, Eq. 9) in LDS
// and every lane expands its windows from there with one vector LDS read per
// MFMA operand.  Weights are the MFMA "A" operand (rows = output channels),
// pixels the "B" operand (columns), so a lane's accumulator registers hold one
// pixel for 16 output channels.
//
// The accumulation order K is free (both operands use the same order), so it
// is chosen per variant to make eight consecutive k contiguous in LDS:
//   planar        (few input channels): K = (ci, ky | kx padded to 8); the input
//                 tile stays planar [ci][row][col]; a lane's eight taps are one
//                 row of the window.
//   channel-block (many input channels): K = (ci/8, ky, kx | ci%8); the input
//                 tile is staged as [ci/8][row][col][8 channels].
//
// Workgroups are persistent: each stages its weights once and then walks tiles
// blockIdx.x, blockIdx.x + gridDim.x, ...  A tile is TM consecutive output
// pixels (row-major within one image) times CB*32 output channels.  Results
// leave through an LDS transpose so that global stores are 16 bytes per lane
// along the contiguous pixel axis of NCHW.
#include "merit_internal.h"

#include <atomic>
#include <type_traits>

namespace merit {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

typedef uint32_t uint32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint32x2 __attribute__((ext_vector_type(2)));

union Frag {
    uint4 u;
    half8 h;
    uint32_t d[4];
};

// One 32x32x16 step: rows of the result are the 32 pixels of `xin`, columns the 32 output
// channels of `wgt` (both fragments: lane l holds row/column l%32, k = 8*(l/32) .. +7).
__device__ __forceinline__ floatx16 mfma16(const Frag &wgt, const Frag &xin, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(xin.h, wgt.h, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack_f16x2(float lo, float hi)
{
    half2v v;
    v.x = (_Float16)lo;       // v_cvt_f16_f32: round to nearest even
    v.y = (_Float16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Touch every 64-byte line of the kernel's argument block (ConvParams + four pointers = five
// lines, and the line after them that holds the grid extents) with the first scalar loads, so that the later ones, issued where their values are needed, hit
// the scalar cache instead of each paying a trip to memory.
static_assert(sizeof(ConvParams) + 4 * sizeof(void *) > 5 * 64 && sizeof(ConvParams) + 4 * sizeof(void *) <= 6 * 64,
              "touch_kernarg_lines covers six 64-byte lines: the argument block must end in the sixth");
__device__ __forceinline__ void touch_kernarg_lines()
{
    typedef const uint32_t __attribute__((address_space(4))) *kernarg_ptr;
    kernarg_ptr ka = (kernarg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
    const uint32_t warm = ka[16] ^ ka[32] ^ ka[48] ^ ka[64] ^ ka[80];   // 80: the grid extents after the pointers
    asm volatile("" ::"s"(warm));
}

// ---------------------------------------------------------------------------
// Epilogue.  Accumulator register r of lane l holds output channel l%32 (within
// its 32-channel block) of pixel 8*(r/4) + 4*(l/32) + r%4 (within its 32-pixel
// block): four consecutive registers are four consecutive pixels of one channel.
// They are rounded to binary16 and written as 8 bytes to LDS, laid out
// outl[channel][pixel]; after a barrier every thread reads runs of 8 pixels of
// one channel and stores them as 16 bytes.  The row pitch of TM/2 + 2 dwords
// spreads the 32 channels of a write over all banks.
// ---------------------------------------------------------------------------
// part 1: accumulators -> LDS staging
// max(v, +0) on two packed binary16 values (v_pk_max_f16: -0 and negative values give +0)
__device__ __forceinline__ uint32_t relu_f16x2(uint32_t v)
{
    const half2v z = {(_Float16)0.0f, (_Float16)0.0f};
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2v, v), z));
}

// add = true: the staging area already holds a tensor of the output's shape in the same
// layout (see stage_residual); it is added to the fp32 sums before the clip and the one
// rounding (the residual layer of Section III-B: a loaded tensor added in PostLoop).  Every
// lane reads exactly the 8 bytes it then overwrites.
template <int CB, int PXW, int NW>
__device__ __forceinline__ void tile_to_lds(floatx16 (&acc)[CB][PXW], uint32_t *outl, int wave, int lane,
                                            bool relu, bool add = false)
{
    constexpr int OP = NW * PXW * 16 + 2;
    const int h = lane >> 5, c32 = lane & 31;
    uint32_t *row = outl + c32 * OP + wave * PXW * 16 + 2 * h;
    if (add) {
        // all reads first: one LDS round trip for the tile
        uint2 rr[CB][PXW][4];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    rr[cb][pb][q] = *reinterpret_cast<const uint2 *>(row + cb * 32 * OP + pb * 16 + 4 * q);
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const half2v r0 = __builtin_bit_cast(half2v, rr[cb][pb][q].x);
                    const half2v r1 = __builtin_bit_cast(half2v, rr[cb][pb][q].y);
                    acc[cb][pb][4 * q] += (float)r0[0];
                    acc[cb][pb][4 * q + 1] += (float)r0[1];
                    acc[cb][pb][4 * q + 2] += (float)r1[0];
                    acc[cb][pb][4 * q + 3] += (float)r1[1];
                }
    }
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint2 v;
                v.x = pack_f16x2(acc[cb][pb][4 * q], acc[cb][pb][4 * q + 1]);
                v.y = pack_f16x2(acc[cb][pb][4 * q + 2], acc[cb][pb][4 * q + 3]);
                if (relu) {        // clipping the rounded value = rounding the clipped value
                    v.x = relu_f16x2(v.x);
                    v.y = relu_f16x2(v.y);
                }
                *reinterpret_cast<uint2 *>(row + cb * 32 * OP + pb * 16 + 4 * q) = v;
            }
}

// part 2: LDS staging -> global, by the NT threads t = 0 .. NT-1 of the storing group
template <int CB, int TM, int NT, bool FULL>
__device__ __forceinline__ void lds_to_global(const ConvParams &p, const uint32_t *outl, uint16_t *__restrict__ y,
                                              int n, int co_base, int m0, int t)
{
    constexpr int OP = TM / 2 + 2;
    const int ohw = p.OH * p.OW;
    const bool vec_ok = (ohw & 7) == 0;
    constexpr int UNITS = CB * 32 * (TM / 8);
    if (!FULL && !vec_ok) {
        // A channel's run of the tile starts at any element of the output: the 16-byte units lie on
        // the output's own 16-byte grid (y itself is 16-byte aligned: the entry points check it; one
        // more unit per channel than the tile has, as the run may straddle), a whole unit is five
        // dwords of the staging row shifted down by one half where its first pixel is odd, and the
        // elements outside every whole unit are stored one by one in a pass of their own (in the same
        // loop every wavefront would take both branches).  As 2-byte stores, 16 bytes apart between
        // lanes, a 53 MB output took 63 us.
        // Tiles that advance by TM - 8 pixels (p.tile_px; they compute TM) own the units that start in
        // their first TM - 8 pixels, the plane's last tile the rest: only a plane's first and last tile
        // then have elements outside every unit.  Tiles that advance by TM have up to 7 at either end.
        const int cnt = min(TM, ohw - m0);
        const bool last = m0 + TM >= ohw, overlap = p.tile_px != TM;
        const int own = (last || !overlap) ? cnt - 7 : p.tile_px;    // a unit is stored if it starts below this pixel
        store_runs_on_grid<TM, NT>(outl, y, ((size_t)n * p.Cout + co_base) * ohw + m0, ohw, cnt, min(CB * 32, p.Cout - co_base),
                                   own, m0 == 0 || !overlap, last || !overlap, t);
        return;
    }
#pragma unroll
    for (int u = t; u < UNITS; u += NT) {
        const int c = u / (TM / 8);
        const int px8 = u - c * (TM / 8);
        const int m = m0 + px8 * 8;
        const int co = co_base + c;
        // FULL: every tile is complete (OH*OW % TM == 0, Cout % (CB*32) == 0), so the stores
        // are unconditional
        if (!FULL && (m >= ohw || co >= p.Cout)) continue;
        const uint2 *src = reinterpret_cast<const uint2 *>(outl + c * OP + px8 * 4);   // 8-byte aligned
        const uint2 a = src[0], b = src[1];
        uint16_t *y0 = y + ((size_t)n * p.Cout + co) * ohw + m;
        // streaming store: written once, not read again here
        uint32x4 v;
        v.x = a.x; v.y = a.y; v.z = b.x; v.w = b.y;
        __builtin_nontemporal_store(v, reinterpret_cast<uint32x4 *>(y0));
    }
}

// Residual layer: the tile of the added tensor r (the output's shape) global -> staging area,
// in the layout and with the thread-to-unit map of lds_to_global.  Called between the two
// barriers that frame a tile's input staging: the previous tile's results have left the area,
// and the barrier before the K loop publishes it.  Every load is issued before the first
// LDS write (one memory round trip); units outside the tensor leave the area untouched
// (their sums are never stored).
template <int CB, int TM, int NT>
__device__ __forceinline__ void stage_residual(const ConvParams &p, uint32_t *outl, const uint16_t *__restrict__ r,
                                               int n, int co_base, int m0, int t)
{
    constexpr int OP = TM / 2 + 2;
    const int ohw = p.OH * p.OW;
    constexpr int UNITS = CB * 32 * (TM / 8);
    constexpr int PER = UNITS / NT;                       // TM/8 and NT are powers of two >= 32
    if ((ohw & 7) == 0) {
        uint32x4 v[PER];
        bool ok[PER];
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int u = t + NT * k;
            const int c = u / (TM / 8);
            const int m = m0 + (u - c * (TM / 8)) * 8;
            ok[k] = m < ohw && co_base + c < p.Cout;
            const size_t off = ok[k] ? ((size_t)n * p.Cout + co_base + c) * ohw + m : 0;
            v[k] = *reinterpret_cast<const uint32x4 *>(r + off);
        }
#pragma unroll
        for (int k = 0; k < PER; ++k) {
            const int u = t + NT * k;
            const int c = u / (TM / 8);
            uint2 *dst = reinterpret_cast<uint2 *>(outl + c * OP + (u - c * (TM / 8)) * 4);
            if (ok[k]) {
                dst[0] = make_uint2(v[k].x, v[k].y);
                dst[1] = make_uint2(v[k].z, v[k].w);
            }
        }
    } else {
        uint16_t *outh = reinterpret_cast<uint16_t *>(outl);
        for (int e = t; e < CB * 32 * TM; e += NT) {
            const int c = e / TM, px = e - c * TM;
            if (m0 + px < ohw && co_base + c < p.Cout)
                outh[c * OP * 2 + px] = r[((size_t)n * p.Cout + co_base + c) * ohw + m0 + px];
        }
    }
}

template <int CB, int PXW, int NW, bool FULL>
__device__ __forceinline__ void store_tile(const ConvParams &p, floatx16 (&acc)[CB][PXW], uint32_t *outl,
                                           uint16_t *__restrict__ y, int n, int co_base, int m0, int tid, bool add)
{
    tile_to_lds<CB, PXW, NW>(acc, outl, tid >> 6, tid & 63, p.relu != 0, add);
    __syncthreads();
    lds_to_global<CB, NW * PXW * 32, NW * 64, FULL>(p, outl, y, n, co_base, m0, tid);
}

// ---------------------------------------------------------------------------
// planar variant
// LDS: [ weights: CB*G2*32 x 16 B ][ 32 B of zeros ][ input: Cin*RHa*pitch halves ]
//      [ output staging ]
// A K-group is one window row (ci, ky), or half of one: its kw taps occupy slots
// front .. front+kw-1 of one 8-slot fragment (kw + front <= 8) or of two adjacent ones
// (up to 16: g = 2 (ci, ky) + part, so lanes 0-31 of a step multiply slots 0-7 and lanes
// 32-63 slots 8-15 of the same row).  front = 0 or 1 is chosen so that the fragment starts
// on an even staged column whenever the column stride is even; unused slots are cleared
// in the data and zero in the weights.
// ---------------------------------------------------------------------------
template <int CB, int PXW, int NW, bool ALIGNED, bool PREFETCH>
__global__ __launch_bounds__(NW * 64, 2) void merit_conv2d_planar(ConvParams p, const uint16_t *__restrict__ x,
                                                             const uint16_t *__restrict__ w,
                                                             const uint16_t *__restrict__ res,
                                                             uint16_t *__restrict__ y)
{
    touch_kernarg_lines();
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *wl = reinterpret_cast<uint4 *>(smem);
    uint8_t *xz = smem + p.lds_w_bytes;                 // 32 zero bytes, then the tile
    uint8_t *xl = xz + 32;
    uint32_t *outl = reinterpret_cast<uint32_t *>(smem + p.lds_o_offset);

    constexpr int NT = NW * 64;                          // threads per workgroup
    constexpr bool FULL = false;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, h = lane >> 5, c32 = lane & 31;
    const int co_base = blockIdx.y * CB * 32;
    const int P8 = p.pitch >> 3;
    const int ohw = p.OH * p.OW;

    // a window row wider than one fragment is two groups (slots 0-7 and 8-15)
    const bool two_parts = p.front + p.kw > 8;
    const int wrows = p.Cin * p.kh;                       // window rows per output channel

    // masks that clear the slots outside [front, front+kw) of a fragment (of this lane's half
    // of the window row when it takes two)
    uint32_t kmask[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int s0 = (two_parts ? h * 8 : 0) + 2 * q - p.front, s1 = s0 + 1;
        kmask[q] = ((s0 >= 0 && s0 < p.kw) ? 0x0000ffffu : 0u) | ((s1 >= 0 && s1 < p.kw) ? 0xffff0000u : 0u);
    }

    const int ntiles = p.N * p.tiles_per_image;
    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2): give every XCD
    // a contiguous run of tiles, so that neighbouring tiles, which share halo rows, meet in
    // one L2.
    const int nwg = (int)gridDim.x;
    const int lw = (nwg % 8 == 0) ? (int)(blockIdx.x % 8) * (nwg / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;

    struct Geom {
        int n, m0, oyA, yA, RH;
    };
    auto geom = [&](int tile) {
        Geom t;
        t.n = (int)fdiv((uint32_t)tile, p.div_tiles);
        t.m0 = (tile - t.n * p.tiles_per_image) * p.tile_px;     // (TM, or TM - 8 where output planes lie off the 16-byte grid)
        t.oyA = (int)fdiv((uint32_t)t.m0, p.div_ow);
        const int mlast = min(t.m0 + p.TM, ohw) - 1;
        const int oyB = (int)fdiv((uint32_t)mlast, p.div_ow);
        t.yA = t.oyA * p.sh - p.ph;
        t.RH = (oyB - t.oyA) * p.sh + p.kh;
        return t;
    };

    // Input staging, 8 halves per unit.  With W % 8 == 0 (and padl == 8) a unit is entirely
    // inside a row or entirely padding, and when one batch of XU units per thread covers the
    // tile the loads of the NEXT tile are issued before the current tile's results are
    // stored, so their latency hides behind the epilogue.
    const int nu = p.Cin * p.RHa * P8;
    const bool vec8 = (p.W & 7) == 0;                     // a unit is one 16-byte load,
    const bool vec_ok = (p.W & 3) == 0;                   // or two of 8 bytes (rows are 8-byte aligned)
    // any other width: 4-byte-aligned loads through one descriptor over the whole tensor (offsets below 2^31)
    const long long xbytes = (long long)p.N * p.Cin * p.H * p.W * 2;
    const bool dw_ok = !vec_ok && xbytes < (1ll << 31);   // (x is 16-byte aligned: the entry points check it)
    // units per thread and batch: 5 when a batch stays in registers across the K loop, else 10 (a
    // batch is one memory round trip)
    constexpr int XU = PREFETCH ? 5 : 10;
    constexpr bool prefetchable = PREFETCH;               // host: W % 8 == 0 and nu <= 5 NT
    uint32x4 pre[XU];
    // unit u = u0 + NT k -> (channel, staged row, column): independent of the tile, so the
    // prefetch path decomposes once; u_off = (ci*H + r)*W + x relative to row yA of the image
    int u_off[XU], u_row[XU];
    bool u_colok[XU], u_col2ok[XU];
    auto decompose = [&](int u0) {
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            const int u = u0 + NT * k;
            const int uc = min(u, nu - 1);
            const int q = (int)fdiv((uint32_t)uc, p.div_pitch8);
            const int c8 = uc - q * P8;
            const int ci = (int)fdiv((uint32_t)q, p.div_rha);
            const int r = q - ci * p.RHa;
            const int xg0 = 8 * c8 - p.padl;
            u_row[k] = r;
            u_colok[k] = u < nu && xg0 >= 0 && xg0 < p.W;
            u_col2ok[k] = xg0 + 4 < p.W;                  // second half of the unit (W % 8 == 4: the row may end between)
            u_off[k] = (ci * p.H + r) * p.W + xg0;
        }
    };
    // The image is read through a buffer descriptor: an offset of 2^31 is past its end, so such
    // a load returns zeros -- padding and rows outside the image need no select on the data (a
    // select right after a load would make the load wait where it is issued), and the two
    // widths stay two different instructions (as plain loads behind a uniform branch the
    // compiler merged them into four 4-byte loads per unit).
    auto issue_loads = [&](const Geom &t) {
        const __amdgpu_buffer_rsrc_t rimg = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(x + (size_t)t.n * p.Cin * p.H * p.W), 0, p.Cin * p.H * p.W * 2, 0x00020000);
        const int yaw = t.yA * p.W;
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            const int gy = t.yA + u_row[k];
            const bool in = u_colok[k] && u_row[k] < t.RH && gy >= 0 && gy < p.H;
            const uint32_t off = in ? (uint32_t)(u_off[k] + yaw) * 2u : 0x80000000u;
            if (PREFETCH || vec8) {
                pre[k] = __builtin_amdgcn_raw_buffer_load_b128(rimg, off, 0, 0);
            } else {
                const uint32x2 a = __builtin_amdgcn_raw_buffer_load_b64(rimg, off, 0, 0);
                const uint32x2 b = __builtin_amdgcn_raw_buffer_load_b64(rimg, (in && u_col2ok[k]) ? off + 8u : 0x80000000u, 0, 0);
                pre[k] = uint32x4{a.x, a.y, b.x, b.y};
            }
        }
    };
    auto commit_loads = [&](int u0) {
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            const int u = u0 + NT * k;
            if (u < nu) reinterpret_cast<uint32x4 *>(xl)[u] = pre[k];
        }
    };

    const uint32_t rowb = (uint32_t)p.pitch * 2u;                 // bytes per staged row
    const uint32_t chb = (uint32_t)p.RHa * rowb;                  // bytes per staged channel
    const uint32_t wrapb = chb - (uint32_t)p.kh * rowb;           // row kh of ci -> row 0 of ci+1
    const bool g_odd = (p.G & 1) != 0;                            // last step: lanes 32-63 have no group
    // which dwords of a fragment hold slots outside [front, front+kw): 1 = first, 2 = last, 3 = any
    // (uniform over the wavefront: with two fragments per row the masks differ between its halves)
    const int mask_mode = two_parts ? 3 : (kmask[0] & kmask[1] & kmask[2] & kmask[3]) == 0xffffffffu ? 0
                          : ((kmask[1] & kmask[2] & kmask[3]) == 0xffffffffu ? 1
                          : ((kmask[0] & kmask[1] & kmask[2]) == 0xffffffffu ? 2 : 3));

    // One tile up to (not including) its stores: stage, multiply, and issue the next tile's
    // input loads.  The caller stores the accumulators afterwards, so that in the steady
    // state the order of memory operations is  loads(t+1), stores(t), [wait loads(t+1)] ...
    // and the wait for the loads does not have to wait for the stores behind them.
    floatx16 acc[CB][PXW];
    auto tile_body = [&](const Geom &T, const Geom &Tn, bool first) {
        __syncthreads();                                  // previous tile fully consumed
        if (p.residual) stage_residual<CB, NW * PXW * 32, NT>(p, outl, res, T.n, co_base, T.m0, tid);
        if (prefetchable) {
            commit_loads(tid);
        } else if (vec_ok) {
            for (int u0 = tid; u0 < nu; u0 += NT * XU) {
                if (!first || u0 != tid) {                 // (the first tile's first batch is in flight already)
                    decompose(u0);
                    issue_loads(T);
                }
                commit_loads(u0);
            }
        } else if (dw_ok) {
            // Rows start at any element: a unit is the 20 bytes from the 4-byte boundary at or below its
            // first element (a 16- and a 4-byte load, UB units in flight per thread), shifted down by one
            // half where it starts odd; what lies past the row's end belongs to the next row and is cleared.
            // (padl == 8: a unit is all padding or starts inside its row.)
            constexpr int UB = 4;
            const __amdgpu_buffer_rsrc_t rall = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(x), 0, (int)xbytes, 0x00020000);
            const int ebase = T.n * p.Cin * p.H * p.W;
            for (int u0 = tid; u0 < nu; u0 += NT * UB) {
                uint32x4 ra[UB];
                uint32_t rb[UB], sh[UB];
                int left[UB], el[UB];                      // elements of the unit inside the row (<= 0: none), first element
                bool whole[UB];                            // both loads lie inside the tensor
#pragma unroll
                for (int k = 0; k < UB; ++k) {
                    const int u = min(u0 + NT * k, nu - 1);
                    const int q = (int)fdiv((uint32_t)u, p.div_pitch8);
                    const int c8 = u - q * P8;
                    const int ci = (int)fdiv((uint32_t)q, p.div_rha);
                    const int r = q - ci * p.RHa;
                    const int gy = T.yA + r;
                    const int xg0 = 8 * c8 - p.padl;
                    const bool in = r < T.RH && gy >= 0 && gy < p.H && xg0 >= 0 && xg0 < p.W;
                    el[k] = ebase + (ci * p.H + gy) * p.W + xg0;
                    left[k] = in ? p.W - xg0 : 0;
                    const uint32_t off = (uint32_t)(el[k] & ~1) * 2u;
                    whole[k] = in && (long long)off + 20 <= xbytes;
                    sh[k] = (uint32_t)(el[k] & 1) * 16u;
                    ra[k] = __builtin_amdgcn_raw_buffer_load_b128(rall, whole[k] ? off : 0x80000000u, 0, 0);
                    rb[k] = __builtin_amdgcn_raw_buffer_load_b32(rall, whole[k] ? off + 16u : 0x80000000u, 0, 0);
                }
#pragma unroll
                for (int k = 0; k < UB; ++k) {
                    const int u = u0 + NT * k;
                    if (u >= nu) break;
                    uint32_t d[4];
                    if (left[k] > 0 && !whole[k]) {        // the tensor's last few elements: one by one
#pragma unroll
                        for (int q = 0; q < 4; ++q) d[q] = 0;
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (e < left[k]) d[e >> 1] |= (uint32_t)x[el[k] + e] << (16 * (e & 1));
                    } else {
                        d[0] = __builtin_amdgcn_alignbit(ra[k].y, ra[k].x, sh[k]);
                        d[1] = __builtin_amdgcn_alignbit(ra[k].z, ra[k].y, sh[k]);
                        d[2] = __builtin_amdgcn_alignbit(ra[k].w, ra[k].z, sh[k]);
                        d[3] = __builtin_amdgcn_alignbit(rb[k], ra[k].w, sh[k]);
#pragma unroll
                        for (int q = 0; q < 4; ++q)
                            d[q] &= (2 * q < left[k] ? 0x0000ffffu : 0u) | (2 * q + 1 < left[k] ? 0xffff0000u : 0u);
                    }
                    reinterpret_cast<uint4 *>(xl)[u] = make_uint4(d[0], d[1], d[2], d[3]);
                }
            }
        } else {
            for (int u = tid; u < nu; u += NT) {
                const int q = (int)fdiv((uint32_t)u, p.div_pitch8);
                const int c8 = u - q * P8;
                const int ci = (int)fdiv((uint32_t)q, p.div_rha);
                const int r = q - ci * p.RHa;
                if (r >= T.RH) continue;
                const int gy = T.yA + r;
                const int xg0 = 8 * c8 - p.padl;
                uint32_t d[4] = {0, 0, 0, 0};
                if (gy >= 0 && gy < p.H && xg0 + 8 > 0 && xg0 < p.W) {
                    const uint16_t *row = x + (((size_t)T.n * p.Cin + ci) * p.H + gy) * p.W;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int xg = xg0 + e;
                        if (xg >= 0 && xg < p.W) d[e >> 1] |= (uint32_t)row[xg] << (16 * (e & 1));
                    }
                }
                reinterpret_cast<uint4 *>(xl)[u] = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
        __syncthreads();

        // ---- per-lane pixel bases ----
        uint32_t pbase[PXW], shift[PXW];
#pragma unroll
        for (int pb = 0; pb < PXW; ++pb) {
            const int m = T.m0 + (wave * PXW + pb) * 32 + c32;
            const int mm = min(m, ohw - 1);
            const int oy = (int)fdiv((uint32_t)mm, p.div_ow);
            const int ox = mm - oy * p.OW;
            const int cs = p.padl - p.pw + ox * p.sw - p.front;       // staged column of slot 0
            pbase[pb] = (uint32_t)((((oy - T.oyA) * p.sh) * p.pitch + (cs & ~1)) * 2) + 32u;
            shift[pb] = (uint32_t)(cs & 1) * 16u;
        }

        // K loop.  Step s feeds group 2s to lanes 0-31 and group 2s+1 to lanes 32-63; a group
        // g = (ci, ky) is one staged row, two rows further per step, so both halves' LDS offsets
        // are advanced incrementally in scalar registers.  Fragments of step s+1 are fetched
        // while the MFMAs of step s run; the first step starts from a zero accumulator.
        // (two fragments per row: both halves walk the same rows, 16 bytes apart, one row per step)
        uint32_t goff[2] = {0u, two_parts ? 16u : ((p.kh == 1) ? chb : rowb)};      // offsets of groups 0 and 1
        int gky[2] = {0, (two_parts || p.kh == 1) ? 0 : 1};
        const int rows_per_step = two_parts ? 1 : 2;
        auto kloop = [&](auto mm_tag) {
            constexpr int MM = decltype(mm_tag)::value;
            // A fetch only reads LDS; the funnel shift and the masks are applied where the fragment is
            // used (done right behind the reads they would make the reads wait where they are issued).
            struct Raw {
                uint32_t d[ALIGNED ? 4 : 5];
            };
            auto load_frags = [&](int s, Frag (&a)[CB], Raw (&r)[PXW]) {
                const uint32_t off = h ? goff[1] : goff[0];
                // group 2s+1 == G: no such row; s == S: the step after the last one, fetched and never
                // used (a fetch under a condition would make every wait in the loop a wait for all)
                const bool dead = (g_odd && h && (s == p.S - 1)) || s >= p.S;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) a[cb].u = wl[cb * p.G2 * 32 + min(s, p.S - 1) * 64 + lane];
#pragma unroll
                for (int pb = 0; pb < PXW; ++pb) {
                    // a dead group reads the zero block (its weights are zero too)
                    const uint32_t addr = dead ? 0u : pbase[pb] + off;
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(xz + addr);
#pragma unroll
                    for (int q = 0; q < (ALIGNED ? 4 : 5); ++q) r[pb].d[q] = src[q];
                }
#pragma unroll
                for (int e = 0; e < 2; ++e) {                         // both halves: two rows on
                    gky[e] += rows_per_step; goff[e] += (uint32_t)rows_per_step * rowb;
                    if (gky[e] >= p.kh) { gky[e] -= p.kh; goff[e] += wrapb; }
                    if (gky[e] >= p.kh) { gky[e] -= p.kh; goff[e] += wrapb; }
                }
            };
            auto mfma_all = [&](Frag (&a)[CB], Raw (&r)[PXW], bool init) {
                Frag b[PXW];
#pragma unroll
                for (int pb = 0; pb < PXW; ++pb) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        b[pb].d[q] = ALIGNED ? r[pb].d[q] : __builtin_amdgcn_alignbit(r[pb].d[ALIGNED ? q : q + 1], r[pb].d[q], shift[pb]);
                    if (MM == 1 || MM == 3) b[pb].d[0] &= kmask[0];
                    if (MM == 3) { b[pb].d[1] &= kmask[1]; b[pb].d[2] &= kmask[2]; }
                    if (MM == 2 || MM == 3) b[pb].d[3] &= kmask[3];
                }
                floatx16 zero;
#pragma unroll
                for (int q = 0; q < 16; ++q) zero[q] = 0.0f;
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int pb = 0; pb < PXW; ++pb) acc[cb][pb] = mfma16(a[cb], b[pb], init ? zero : acc[cb][pb]);
            };
            Frag a0[CB], a1[CB];
            Raw r0[PXW], r1[PXW];
            load_frags(0, a0, r0);
            load_frags(1, a1, r1);
            mfma_all(a0, r0, true);                                   // the first step starts from zero
            int s = 1;                                                // a1/r1 hold step s
            // (the fences keep the scheduler from sinking a fetch below the MFMAs it is meant to run under)
            for (; s + 2 <= p.S; s += 2) {
                load_frags(s + 1, a0, r0);
                __builtin_amdgcn_sched_barrier(0);
                mfma_all(a1, r1, false);
                __builtin_amdgcn_sched_barrier(0);
                load_frags(s + 2, a1, r1);
                __builtin_amdgcn_sched_barrier(0);
                mfma_all(a0, r0, false);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (s < p.S) mfma_all(a1, r1, false);
        };
        if (mask_mode == 0) kloop(std::integral_constant<int, 0>{});
        else if (mask_mode == 1) kloop(std::integral_constant<int, 1>{});
        else if (mask_mode == 2) kloop(std::integral_constant<int, 2>{});
        else kloop(std::integral_constant<int, 3>{});

        // next tile's input loads (unconditionally: the last tile re-loads itself, which keeps
        // the loaded registers free of copies)
        if (prefetchable) issue_loads(Tn);
    };

    int tile = lw;                                        // < ntiles: the grid never exceeds it
    Geom T = geom(tile);
    Geom Tn = geom(min(tile + nwg, ntiles - 1));
    // the first tile's (first batch of) input loads go out before the weights are fetched: one
    // memory round trip for both
    if (prefetchable || vec_ok) {
        decompose(tid);
        issue_loads(T);
    }

    // ---- weights, once per workgroup: unit = (local output channel, group) ----
    const int units = CB * 32 * p.G2;
    const int nco = min(CB * 32, p.Cout - co_base);
    const int wtotal = nco * wrows * p.kw;                // halves of this workgroup's block: contiguous
    const long long wbytes = (long long)p.Cout * wrows * p.kw * 2;
    if (wtotal * 2 + 64 <= p.lds_total - p.lds_w_bytes - 32 && wbytes < (1ll << 31)) {
        // The block fits the (not yet used) tile area: it is parked there as it lies in memory, with
        // 16-byte loads, and the fragments are
        // cut out of LDS -- five dwords around a fragment's 8 slots, shifted by one half if needed.
        // As 2-byte gathers from global memory the same took three to four times as long.
        const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(w), 0, (int)wbytes, 0x00020000);
        const uint32_t base = (uint32_t)co_base * (uint32_t)(wrows * p.kw) * 2u;      // a multiple of 64
        // whole 16-byte vectors inside the tensor; the last block's last few halves (a load that is
        // only partly in range returns zeros for all of it) are fetched one by one
        const int nvec = min((wtotal * 2 + 15) >> 4, (int)((wbytes - (long long)base) >> 4));
        if (tid < 8 && nvec * 8 + tid < wtotal)
            reinterpret_cast<uint16_t *>(xl)[nvec * 8 + tid] = w[(size_t)co_base * (size_t)(wrows * p.kw) + nvec * 8 + tid];
        constexpr int WB = 12;
        for (int i0 = tid; i0 < nvec; i0 += NT * WB) {
            uint32x4 v[WB];
#pragma unroll
            for (int k = 0; k < WB; ++k) {
                const int i = i0 + NT * k;
                v[k] = __builtin_amdgcn_raw_buffer_load_b128(rw, i < nvec ? base + 16u * (uint32_t)i : 0x80000000u, 0, 0);   // (2^31: out of range, no load)
            }
#pragma unroll
            for (int k = 0; k < WB; ++k) {
                const int i = i0 + NT * k;
                if (i < nvec) reinterpret_cast<uint32x4 *>(xl)[i] = v[k];
            }
        }
        __syncthreads();
        const uint32_t *rawd = reinterpret_cast<const uint32_t *>(xl);
        // A thread keeps its channel and walks the groups: consecutive lanes take consecutive
        // channels of one group, so their 16-byte writes are adjacent (lanes along the groups would
        // write 512 bytes apart, all into the same four banks).  Four fragments per batch: every LDS
        // read of a batch is issued before the first use (a lone wavefront per SIMD cannot hide
        // the latency otherwise: 3.4 us for the 66 groups of an 11x11 window on 3 channels).
        constexpr int GSTEP = NT / (CB * 32);               // groups between a thread's units: 4, 8 or 16
        constexpr int WQ = 4;
        const int col = tid & (CB * 32 - 1);
        const int g0 = tid / (CB * 32);
        const int part = two_parts ? g0 & 1 : 0;           // GSTEP is even: a thread stays in its half of the row
        // valid slots of this thread's fragments: bit t of `valid` = slot t holds a tap; one mask per dword
        const uint32_t valid = ((((1u << p.kw) - 1u) << p.front) >> (8 * part)) & 0xffu;
        uint32_t wm[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) wm[q] = ((valid >> (2 * q)) & 1u) * 0x0000ffffu | ((valid >> (2 * q + 1)) & 1u) * 0xffff0000u;
        const int dstart = (two_parts ? GSTEP / 2 : GSTEP) * p.kw;
        int start = (col * wrows + (two_parts ? g0 >> 1 : g0)) * p.kw + part * 8 - p.front;        // >= -1: inside LDS
        int dst = ((col >> 5) * p.G2 + g0) * 32 + (col & 31);
        for (int g = g0; g < p.G2; g += WQ * GSTEP) {
            uint32_t d[WQ][5];
            uint32_t sh[WQ];
            bool ok[WQ];
#pragma unroll
            for (int k = 0; k < WQ; ++k) {
                ok[k] = col < nco && g + k * GSTEP < p.G;
                const int st = ok[k] ? start + k * dstart : 0;
                sh[k] = (uint32_t)(st & 1) * 16u;
                const uint32_t *r = rawd + (st >> 1);
#pragma unroll
                for (int q = 0; q < 5; ++q) d[k][q] = r[q];
            }
#pragma unroll
            for (int k = 0; k < WQ; ++k) {
                uint32_t o[4];
                const uint32_t okm = ok[k] ? 0xffffffffu : 0u;      // (no branch: what was read for a unit that is not there is inside LDS)
#pragma unroll
                for (int q = 0; q < 4; ++q) o[q] = __builtin_amdgcn_alignbit(d[k][q + 1], d[k][q], sh[k]) & wm[q] & okm;
                if (g + k * GSTEP < p.G2) wl[dst + k * GSTEP * 32] = make_uint4(o[0], o[1], o[2], o[3]);
            }
            start += WQ * dstart;
            dst += WQ * GSTEP * 32;
        }
        if (tid < 8) reinterpret_cast<uint32_t *>(xz)[tid] = 0;
    } else {
        // batches of WU units: all global loads of a batch are issued before the first LDS
        // write, so a batch costs one memory round trip
        constexpr int WU = 6;
        for (int u0 = tid; u0 < units; u0 += NT * WU) {
            uint16_t hv[WU][8];
            bool ok[WU];
#pragma unroll
            for (int k = 0; k < WU; ++k) {
                const int u = min(u0 + NT * k, units - 1);
                const int col = (int)fdiv((uint32_t)u, p.div_g2);
                const int g = u - col * p.G2;
                const int co = co_base + col;
                ok[k] = co < p.Cout && g < p.G;
                const int row = two_parts ? g >> 1 : g;     // (ci, ky)
                const int tap0 = (two_parts ? (g & 1) * 8 : 0) - p.front;      // tap in slot 0 of this fragment
                const uint16_t *src = w + (ok[k] ? ((size_t)co * wrows + row) * p.kw : 0);
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    const int tap = tap0 + t;
                    hv[k][t] = (tap >= 0 && tap < p.kw) ? src[tap] : (uint16_t)0;
                }
            }
#pragma unroll
            for (int k = 0; k < WU; ++k) {
                const int u = u0 + NT * k;
                if (u >= units) break;
                const int col = (int)fdiv((uint32_t)u, p.div_g2);
                const int g = u - col * p.G2;
                uint32_t d[4] = {0, 0, 0, 0};
                if (ok[k]) {
#pragma unroll
                    for (int t = 0; t < 8; ++t) d[t >> 1] |= (uint32_t)hv[k][t] << (16 * (t & 1));
                }
                wl[((col >> 5) * p.G2 + g) * 32 + (col & 31)] = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
        if (tid < 8) reinterpret_cast<uint32_t *>(xz)[tid] = 0;
    }

    tile_body(T, Tn, true);
    for (tile += nwg; tile < ntiles; tile += nwg) {
        store_tile<CB, PXW, NW, FULL>(p, acc, outl, y, T.n, co_base, T.m0, tid, p.residual != 0);
        T = Tn;
        Tn = geom(min(tile + nwg, ntiles - 1));
        tile_body(T, Tn, false);
    }
    store_tile<CB, PXW, NW, FULL>(p, acc, outl, y, T.n, co_base, T.m0, tid, p.residual != 0);
}

// ---------------------------------------------------------------------------
// planar variant, wave-specialised (8 wavefronts per workgroup, one workgroup per CU)
// LDS: [ weights ][ 32 B zeros ][ input tile A ][ input tile B ][ out staging A ][ out staging B ]
//
// Wavefronts 0-3 only multiply: K loop of tile i out of input buffer i%2, then the rounded
// results into out staging i%2.  They never touch global memory, and they keep every weight
// fragment in registers, so the K loop reads only input fragments from LDS.  The K loop is
// SU steps without a branch (template parameter, S <= SU <= S+2).
// Wavefronts 4-5 only load: in iteration i they write the (already loaded) input of tile
// i+1 into buffer (i+1)%2 and issue the global loads of tile i+2.  Wavefronts 6-7 only
// store: the results of tile i-1 from out staging (i-1)%2 to global memory.
// One barrier per iteration hands the buffers over; memory latency lives in the mover
// wavefronts and is covered by a whole K loop of the multiplier wavefronts.
// Needs W % 8 == 0, OH*OW % 8 == 0, tensors below 2 GiB and at most 10 staging units per
// loading thread.
//
// POOL: the convolution feeds a 3x3 / stride 2 / padding 1 max pooling and only the pooled
// tensor is written (the fused CONV+Pool layers of the per-layer table in Section VI-C).
// A workgroup owns a band of PB pooled rows of one image; its tile i is the pair of
// convolution rows 2r, 2r+1 with r = band*PB - 1 + i (two whole rows of OW <= 128 pixels in
// the 256-pixel tile).  Pooled row r needs rows 2r-1, 2r, 2r+1: the storing wavefronts take
// the element-wise maximum of both rows of a tile and the previous tile's second row (carried
// in registers: every unit of 8 pooled pixels belongs to one thread for the whole band), then
// the 3-maxima along the row at stride 2, and store 8 pooled pixels per unit.  Tile 0 of a
// band only fills the carry (-inf above the image).  All maxima are v_pk_maximum3_f16.
// ---------------------------------------------------------------------------
// elementwise maximum of three binary16 pairs: one v_pk_maximum3_f16
__device__ __forceinline__ uint32_t pkmax3_f16x2(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_bit_cast(
        uint32_t, __builtin_elementwise_maximum(
                      __builtin_elementwise_maximum(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b)),
                      __builtin_bit_cast(half2v, c)));
}

// column-wise 3-maxima of one row at stride 2: d[k] = columns 2k, 2k+1 of the unit (binary16
// pairs), left = the pair before d[0]; result = 8 pooled pixels m_k = max(col 2k-1, 2k, 2k+1),
// two at a time: { m_2j, m_2j+1 } = max( {col 4j, col 4j+2}, {col 4j+1, col 4j+3}, {col 4j-1, col 4j+1} )
__device__ __forceinline__ uint32x4 row_max3_s2(uint32_t left, const uint32_t (&d)[8])
{
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint32_t before = j == 0 ? left : d[2 * j - 1];
        const uint32_t ev = __builtin_amdgcn_perm(d[2 * j + 1], d[2 * j], 0x05040100u);
        const uint32_t od = __builtin_amdgcn_perm(d[2 * j + 1], d[2 * j], 0x07060302u);
        const uint32_t pv = __builtin_amdgcn_perm(d[2 * j], before, 0x07060302u);
        o[j] = pkmax3_f16x2(ev, od, pv);
    }
    uint32x4 r;
    r.x = o[0]; r.y = o[1]; r.z = o[2]; r.w = o[3];
    return r;
}

template <int CB, bool ALIGNED, int SU, bool POOL, bool UNAL = false>
__global__ __launch_bounds__(512, 1) void merit_conv2d_planar_ws(ConvParams p, const uint16_t *__restrict__ x,
                                                                const uint16_t *__restrict__ w,
                                                                const uint16_t *__restrict__ /* no residual layer here */,
                                                                uint16_t *__restrict__ y)
{
    constexpr int PXW = 2, NWC = 4, TM = NWC * PXW * 32, NTG = 128;    // loading / storing group = 2 wavefronts
    touch_kernarg_lines();
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *wl = reinterpret_cast<uint4 *>(smem);
    uint8_t *xz = smem + p.lds_w_bytes;                 // 32 zero bytes, then the two tiles
    const uint32_t xstride = (uint32_t)p.lds_x_bytes;   // multiple of 16
    uint8_t *outl0 = smem + p.lds_o_offset;
    const uint32_t ostride = (uint32_t)p.lds_o_bytes;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, h = lane >> 5, c32 = lane & 31;
    const bool mover = wave >= NWC;
    const bool loader = wave >= NWC && wave < NWC + 2;  // wavefronts 4-5 load, 6-7 store
    const int t = tid & (NTG - 1);                      // index inside the loading / storing group
    const int cwave = wave & (NWC - 1);
    const int co_base = blockIdx.y * CB * 32;
    const int P8 = p.pitch >> 3;
    const int ohw = p.OH * p.OW;

    // ---- weights, once per workgroup (all 512 threads) ----
    // The (CB*32) x G x kw block of this workgroup's output channels is contiguous in global
    // memory (at most 3 x 512 16-byte vectors): request it before anything else, so that the
    // first memory round trip of the kernel runs under the index set-up below.  It is parked in
    // LDS (the out staging area is still free) and rearranged into fragments from there.
    const int nco = min(CB * 32, p.Cout - co_base);
    const int wrow = p.G * p.kw;                        // halves per output channel
    const int wtotal = nco * wrow;
    const int wvec = wtotal >> 3;
    constexpr int WV = 3;
    // co_base % 32 == 0 keeps the block 16-byte aligned; it holds at least one vector
    const uint4 *wsrc = reinterpret_cast<const uint4 *>(w + (size_t)co_base * wrow);
    const uint4 wraw0 = wsrc[min(tid, wvec - 1)];
    const uint4 wraw1 = wsrc[min(tid + 512, wvec - 1)];
    const uint4 wraw2 = wsrc[min(tid + 1024, wvec - 1)];
    auto weights_park = [&]() {
        uint16_t *rawh = reinterpret_cast<uint16_t *>(outl0);
        if (tid < wvec) reinterpret_cast<uint4 *>(rawh)[tid] = wraw0;
        if (tid + 512 < wvec) reinterpret_cast<uint4 *>(rawh)[tid + 512] = wraw1;
        if (tid + 1024 < wvec) reinterpret_cast<uint4 *>(rawh)[tid + 1024] = wraw2;
        const uint16_t *src = w + (size_t)co_base * wrow;
        for (int e = (wvec << 3) + tid; e < wtotal; e += 512) rawh[e] = src[e];
    };
    // masks that clear the slots outside [front, front+kw) of a fragment
    uint32_t kmask[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int s0 = 2 * q - p.front, s1 = 2 * q + 1 - p.front;
        kmask[q] = ((s0 >= 0 && s0 < p.kw) ? 0x0000ffffu : 0u) | ((s1 >= 0 && s1 < p.kw) ? 0xffff0000u : 0u);
    }
    auto weights_frag = [&]() {
        // unit = (local channel, group): its kw taps start at half (col*G + g)*kw of the parked
        // block and go to slots front .. front+kw-1.  Five dwords around them are read whole
        // (what lies outside the block is inside LDS and masked) and shifted by one half if needed.
        const uint32_t *rawd = reinterpret_cast<const uint32_t *>(outl0);
        const int units = CB * 32 * p.G2;                 // at most 3 per thread
        uint32_t d[WV][5];
        uint32_t sh[WV];
        int dst[WV];
        bool ok[WV];
#pragma unroll
        for (int k = 0; k < WV; ++k) {                     // every LDS read before the first use
            const int u = min(tid + 512 * k, units - 1);
            const int col = (int)fdiv((uint32_t)u, p.div_g2);
            const int g = u - col * p.G2;
            ok[k] = col < nco && g < p.G;
            const int start = (ok[k] ? (col * p.G + g) * p.kw : 0) - p.front;     // >= -1
            dst[k] = ((col >> 5) * p.G2 + g) * 32 + (col & 31);
            sh[k] = (uint32_t)(start & 1) * 16u;
            const uint32_t *r = rawd + (start >> 1);
#pragma unroll
            for (int q = 0; q < 5; ++q) d[k][q] = r[q];
        }
#pragma unroll
        for (int k = 0; k < WV; ++k) {
            uint32_t o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                o[q] = ok[k] ? (__builtin_amdgcn_alignbit(d[k][q + 1], d[k][q], sh[k]) & kmask[q]) : 0u;
            if (tid + 512 * k < units) wl[dst[k]] = make_uint4(o[0], o[1], o[2], o[3]);
        }
        if (tid < 8) reinterpret_cast<uint32_t *>(xz)[tid] = 0;
    };

    const int ntiles = p.N * p.tiles_per_image;
    const int nwg = (int)gridDim.x;
    const int lw = (nwg % 8 == 0) ? (int)(blockIdx.x % 8) * (nwg / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    // POOL: workgroup lw = (image, band); tile i = convolution row pair rp0 + i
    const int band_n = POOL ? (int)fdiv((uint32_t)lw, p.div_nb) : 0;
    const int band = POOL ? lw - band_n * p.NB : 0;
    const int rp0 = band * p.PB - 1;
    const int K = POOL ? min(p.PB, p.PH - band * p.PB) + 1
                       : (ntiles - lw + nwg - 1) / nwg;   // tiles of this workgroup (>= 1)

    struct Geom {
        int n, m0, oyA, yA, RH;
    };
    auto geom = [&](int i) {                              // i-th tile of this workgroup, clamped
        if constexpr (POOL) {
            Geom g;
            g.n = band_n;
            g.m0 = 0;
            g.oyA = 2 * (rp0 + min(i, K - 1));            // -2 for the tile above the image: all zeros
            g.yA = g.oyA * p.sh - p.ph;
            g.RH = p.sh + p.kh;
            return g;
        }
        const int tile = lw + min(i, K - 1) * nwg;
        Geom g;
        g.n = (int)fdiv((uint32_t)tile, p.div_tiles);
        g.m0 = (tile - g.n * p.tiles_per_image) * (UNAL ? p.tile_px : p.TM);
        g.oyA = (int)fdiv((uint32_t)g.m0, p.div_ow);
        const int mlast = min(g.m0 + p.TM, ohw) - 1;
        const int oyB = (int)fdiv((uint32_t)mlast, p.div_ow);
        g.yA = g.oyA * p.sh - p.ph;
        g.RH = (oyB - g.oyA) * p.sh + p.kh;
        return g;
    };

    // ---- mover state: staging units of this thread (tile-independent decomposition) ----
    // Global memory is reached through buffer descriptors: an offset of 2^31 is past the end
    // of either tensor, so such a load returns zeros and such a store is dropped.  Padding,
    // halo rows outside the image and partial tiles need no branch and no select on the data.
    constexpr uint32_t OOB = 0x80000000u;
    const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t *>(x), 0, (int)((size_t)p.N * p.Cin * p.H * p.W * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t ry = __builtin_amdgcn_make_buffer_rsrc(
        y, 0, (int)((size_t)p.N * p.Cout * (POOL ? p.PH * p.PW : ohw) * 2), 0x00020000);
    // Loading thread t owns 16-byte column chunk t % 2^lgc of the staged rows
    // q = t / 2^lgc + (128 >> lgc) k  (q = ci*RHa + r; 2^lgc >= chunks per row), so that a
    // thread's column tests are shared by all its units and only q needs a division.
    constexpr int XU = 10;
    uint32x4 pre[XU];
    int u_off2[XU], u_row[XU], u_lds[XU];                 // byte offset in the image at yA = 0; staged row
    bool u_live[XU];
    const int lgc = p.lg_chunks;
    const int ld_c8 = t & ((1 << lgc) - 1);
    const int ld_xg0 = 8 * ld_c8 - p.padl;
    const bool ld_colok = ld_xg0 >= 0 && ld_xg0 < p.W;    // else: padding columns, zero-filled
    if (loader) {
        const int nq = p.Cin * p.RHa;
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            const int q = (t >> lgc) + (NTG >> lgc) * k;
            const int qc = min(q, nq - 1);
            const int ci = (int)fdiv((uint32_t)qc, p.div_rha);
            const int r = qc - ci * p.RHa;
            u_row[k] = r;
            u_live[k] = q < nq && ld_c8 < P8;
            u_off2[k] = ((ci * p.H + r) * p.W + ld_xg0) * 2;
            u_lds[k] = (qc * P8 + min(ld_c8, P8 - 1)) * 16;
        }
    }
    // UNAL (rows that start on any element: W % 8 != 0): a unit is the 20 bytes from the 4-byte
    // boundary at or below its first element, one 16- and one 4-byte load, shifted down by a half
    // where it starts odd; what lies past the row's end (the next row's first pixels) is cleared.
    // A load only partly in range returns zeros for all of it, so the unit whose 20 bytes would
    // cross the tensor's end (at most one per thread) is fetched element by element when it is written.
    uint32_t pre4[UNAL ? XU : 1], u_sh[UNAL ? XU : 1];
    uint32_t cmask[4];                                    // the halves of this thread's column chunk inside the row
#pragma unroll
    for (int q = 0; q < 4; ++q)
        cmask[q] = (ld_xg0 + 2 * q < p.W ? 0x0000ffffu : 0u) | (ld_xg0 + 2 * q + 1 < p.W ? 0xffff0000u : 0u);
    const uint32_t xbytes = (uint32_t)((size_t)p.N * p.Cin * p.H * p.W * 2);
    uint32_t tail_voff = OOB;
    int tail_lds = 0;
    auto issue_loads = [&](const Geom &g) {
        const uint32_t soff = (uint32_t)g.n * (uint32_t)(p.Cin * p.H * p.W * 2);
        const int yaw2 = g.yA * p.W * 2;
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            const uint32_t gy = (uint32_t)(g.yA + u_row[k]);
            const int ok = (int)ld_colok & (int)(u_row[k] < g.RH) & (int)(gy < (uint32_t)p.H);
            if constexpr (UNAL) {
                const uint32_t ab = soff + (uint32_t)(u_off2[k] + yaw2);      // first element, from the tensor's start
                const uint32_t al = ab & ~3u;
                const bool whole = al + 20u <= xbytes;
                u_sh[k] = (ab & 2u) * 8u;
                pre[k] = __builtin_amdgcn_raw_buffer_load_b128(rx, (ok && whole) ? al : OOB, 0, 0);
                pre4[k] = __builtin_amdgcn_raw_buffer_load_b32(rx, (ok && whole) ? al + 16u : OOB, 0, 0);
                if (ok && !whole && u_live[k]) {
                    tail_voff = ab;
                    tail_lds = u_lds[k];
                }
            } else {
                const uint32_t voff = ok ? (uint32_t)(u_off2[k] + yaw2) : OOB;
                pre[k] = __builtin_amdgcn_raw_buffer_load_b128(rx, voff, soff, 0);
            }
        }
    };
    auto commit_loads = [&](uint8_t *xl) {
#pragma unroll
        for (int k = 0; k < XU; ++k) {
            if constexpr (UNAL) {
                uint32x4 d;
                d.x = __builtin_amdgcn_alignbit(pre[k].y, pre[k].x, u_sh[k]) & cmask[0];
                d.y = __builtin_amdgcn_alignbit(pre[k].z, pre[k].y, u_sh[k]) & cmask[1];
                d.z = __builtin_amdgcn_alignbit(pre[k].w, pre[k].z, u_sh[k]) & cmask[2];
                d.w = __builtin_amdgcn_alignbit(pre4[k], pre[k].w, u_sh[k]) & cmask[3];
                if (u_live[k]) *reinterpret_cast<uint32x4 *>(xl + u_lds[k]) = d;
            } else {
                if (u_live[k]) *reinterpret_cast<uint32x4 *>(xl + u_lds[k]) = pre[k];
            }
        }
        if constexpr (UNAL) {
            if (tail_voff != OOB) {
                uint32_t d[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t hv = __builtin_amdgcn_raw_buffer_load_b16(rx, ld_xg0 + e < p.W ? tail_voff + 2u * e : OOB, 0, 0);
                    d[e >> 1] |= (hv & 0xffffu) << (16 * (e & 1));
                }
                uint32x4 dv;
                dv.x = d[0]; dv.y = d[1]; dv.z = d[2]; dv.w = d[3];
                *reinterpret_cast<uint32x4 *>(xl + tail_lds) = dv;
                tail_voff = OOB;
            }
        }
    };
    // results: thread t stores 8 pixels of channels t/32 + 4k, k = 0 .. CB*8-1
    constexpr int OPW = TM / 2 + 2;                       // out staging pitch in dwords
    const int st_c0 = t >> 5, st_px = (t & 31) * 8;
    const uint32_t st_voff = (uint32_t)(st_c0 * ohw + st_px) * 2u;
    const int st_nc = p.Cout - co_base - st_c0;           // channel t/32 + 4k exists iff 4k < st_nc
    auto store_tile_ws = [&](int i) {
        const Geom P = geom(i);
        const uint32_t *src = reinterpret_cast<const uint32_t *>(outl0 + (i & 1) * ostride) + st_c0 * OPW + (t & 31) * 4;
        const uint32_t soff = (uint32_t)(((size_t)P.n * p.Cout + co_base) * ohw + P.m0) * 2u;
        const bool mok = P.m0 + st_px < ohw;
#pragma unroll
        for (int k = 0; k < CB * 8; ++k) {
            const uint2 a = *reinterpret_cast<const uint2 *>(src + k * 4 * OPW);
            const uint2 b = *reinterpret_cast<const uint2 *>(src + k * 4 * OPW + 2);
            uint32x4 v;
            v.x = a.x; v.y = a.y; v.z = b.x; v.w = b.y;
            // The whole offset goes into the vector register and the scalar offset stays 0: for
            // a 16-byte buffer store WITH a scalar offset register the compiler leaves no gap
            // before the next instruction that overwrites the data registers, and on this chip
            // that instruction was seen to win the race (first dword of the run corrupted).
            const uint32_t voff = (mok && 4 * k < st_nc) ? st_voff + soff + (uint32_t)(k * 4 * ohw * 2) : OOB;
            // cache policy "sc0 nt": results are written once and not read again by this kernel;
            // streaming them keeps the L2 from collecting dirty lines that the end of the
            // kernel then has to write back all at once
            __builtin_amdgcn_raw_buffer_store_b128(v, ry, voff, 0, 3);
        }
    };

    // UNAL, output planes that start on any element (OH*OW % 8 != 0): the 16-byte store units lie on
    // the output's own 16-byte grid.  Tiles advance by TM - 8 pixels and compute TM, so every unit of a
    // channel's plane lies inside the tile that owns its first pixel (the first TM - 8 of a tile; the
    // plane's last tile owns the rest): lane j of a channel stores the unit that starts `head + 8j`
    // pixels into the tile's run -- five dwords of the staging row, shifted down by a half where that
    // pixel is odd.  Only a plane's first and last tile have elements outside every unit (up to 7 each,
    // shared 16-byte units with the neighbouring planes): 2-byte stores, 16 lanes per channel.  (With
    // tiles that end where the next begins -- p.tile_px == TM, taken where the extra tiles would cost the
    // grid another round -- every tile has such ends: 2.5 million 2-byte stores into lines that other
    // workgroups write, 36 us instead of 31 on a 91 MB output.)
    auto store_tile_ws_grid = [&](int i) {
        const Geom P = geom(i);
        const uint32_t *src0 = reinterpret_cast<const uint32_t *>(outl0 + (i & 1) * ostride);
        const uint32_t a0 = (uint32_t)(((size_t)P.n * p.Cout + co_base) * ohw + P.m0);      // element index (bytes < 2^31)
        const int cnt = min(TM, ohw - P.m0);
        const bool last = P.m0 + TM >= ohw, overlap = p.tile_px != TM;
        const int own = (last || !overlap) ? cnt - 7 : TM - 8;  // a unit is stored if it starts below this pixel of the tile
        const bool heads = P.m0 == 0 || !overlap, tails = last || !overlap;
        const int j = t & 31;
#pragma unroll
        for (int k = 0; k < CB * 8; ++k) {
            const int c = st_c0 + 4 * k;
            const uint32_t a = a0 + (uint32_t)(c * ohw);
            const int px0 = (int)((8u - (a & 7u)) & 7u) + 8 * j;
            const int pxr = max(min(px0, cnt - 8), 0);         // (a unit that is not stored reads inside the row all the same)
            const int d0 = pxr >> 1;
            const uint32_t *r = src0 + c * OPW + (d0 & ~1);     // 8-byte aligned
            const uint2 A = *reinterpret_cast<const uint2 *>(r);
            const uint2 B = *reinterpret_cast<const uint2 *>(r + 2);
            const uint2 C = *reinterpret_cast<const uint2 *>(r + 4);
            const bool odd = (d0 & 1) != 0;
            const uint32_t w0 = odd ? A.y : A.x, w1 = odd ? B.x : A.y, w2 = odd ? B.y : B.x, w3 = odd ? C.x : B.y,
                           w4 = odd ? C.y : C.x;
            const uint32_t sh = (uint32_t)(pxr & 1) * 16u;
            uint32x4 v;
            v.x = __builtin_amdgcn_alignbit(w1, w0, sh);
            v.y = __builtin_amdgcn_alignbit(w2, w1, sh);
            v.z = __builtin_amdgcn_alignbit(w3, w2, sh);
            v.w = __builtin_amdgcn_alignbit(w4, w3, sh);
            const uint32_t voff = (4 * k < st_nc && px0 < own) ? (a + (uint32_t)px0) * 2u : OOB;
            __builtin_amdgcn_raw_buffer_store_b128(v, ry, voff, 0, 3);
        }
        if (heads || tails) {
            const int ec0 = t >> 4, kq = t & 7;
#pragma unroll
            for (int k = 0; k < CB * 4; ++k) {
                const int c = ec0 + 8 * k;
                const uint32_t a = a0 + (uint32_t)(c * ohw);
                const int head = min(cnt, (int)((8u - (a & 7u)) & 7u));
                // lanes 0-7 of a channel: the pixels before the first unit of the plane's first tile;
                // lanes 8-15: the pixels behind the last unit of its last tile
                const int px = (t & 8) ? (tails ? head + ((cnt - head) & ~7) + kq : cnt) : ((heads && kq < head) ? kq : cnt);
                const uint16_t hv = reinterpret_cast<const uint16_t *>(src0 + c * OPW)[min(px, TM - 1)];
                const uint32_t voff = (c < p.Cout - co_base && px < cnt) ? (a + (uint32_t)px) * 2u : OOB;
                __builtin_amdgcn_raw_buffer_store_b16(hv, ry, voff, 0, 3);
            }
        }
    };

    // POOL: thread t owns the units u = t + 128k (u = channel * pw8 + 8-pixel unit of the pooled row)
    constexpr int PU = 2 * CB;                            // CB*32 channels x at most 8 units / 128 threads
    constexpr uint32_t NEG = 0xFC00FC00u;                 // two binary16 -inf
    int pl_src[PU];                                       // dword of the unit's first column pair in a staged tile
    uint32_t pl_y[PU];                                    // byte offset of the unit inside an image's pooled rows
    bool pl_live[PU], pl_left[PU];
    uint32_t carry[PU][9];                                // previous tile's second row: 8 pairs + the pair before
    if constexpr (POOL) {
        const int units = CB * 32 * p.pw8;
#pragma unroll
        for (int k = 0; k < PU; ++k) {
            const int u = t + NTG * k;
            const int uc = min(u, units - 1);
            const int c = (int)fdiv((uint32_t)uc, p.div_pw8);
            const int ux = uc - c * p.pw8;
            pl_src[k] = c * OPW + 8 * ux;
            pl_y[k] = (uint32_t)(c * p.PH * p.PW + 8 * ux) * 2u;
            pl_live[k] = u < units && c < p.Cout - co_base;
            pl_left[k] = ux > 0;
#pragma unroll
            for (int q = 0; q < 9; ++q) carry[k][q] = NEG;
        }
    }
    auto pool_tile_ws = [&](int i) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(outl0 + (i & 1) * ostride);
        const int py = rp0 + i;                           // pooled row this tile completes (i >= 1)
        const uint32_t soff = (uint32_t)((((size_t)band_n * p.Cout + co_base) * p.PH + max(py, 0)) * p.PW) * 2u;
        const bool above = py < 0;                        // the tile above the image: its rows count as -inf
        const int rowd = p.OW >> 1;                       // dwords per convolution row
#pragma unroll
        for (int k = 0; k < PU; ++k) {
            const uint32_t *ra = src + pl_src[k];
            const uint32_t *rb = ra + rowd;
            uint32_t a[8], b[8];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint2 va = *reinterpret_cast<const uint2 *>(ra + 2 * q);
                const uint2 vb = *reinterpret_cast<const uint2 *>(rb + 2 * q);
                a[2 * q] = va.x; a[2 * q + 1] = va.y;
                b[2 * q] = vb.x; b[2 * q + 1] = vb.y;
            }
            const int lo = pl_left[k] ? -1 : 0;           // column -1 is padding (-inf)
            const uint32_t la_raw = ra[lo], lb_raw = rb[lo];
            const uint32_t la = pl_left[k] ? la_raw : NEG;
            const uint32_t lb = pl_left[k] ? lb_raw : NEG;
            uint32_t m[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) m[q] = pkmax3_f16x2(a[q], b[q], carry[k][q]);
            const uint32_t ml = pkmax3_f16x2(la, lb, carry[k][8]);
            const uint32x4 v = row_max3_s2(ml, m);
#pragma unroll
            for (int q = 0; q < 8; ++q) carry[k][q] = above ? NEG : b[q];
            carry[k][8] = above ? NEG : lb;
            // whole offset in the vector register, scalar offset 0 (see store_tile_ws)
            const uint32_t voff = (i >= 1 && pl_live[k]) ? pl_y[k] + soff : OOB;
            __builtin_amdgcn_raw_buffer_store_b128(v, ry, voff, 0, 3);
        }
    };

    // first input tile requested as early as its addresses are known
    if (loader) issue_loads(geom(0));

    const uint32_t rowb = (uint32_t)p.pitch * 2u;
    const uint32_t chb = (uint32_t)p.RHa * rowb;
    const int mask_mode = (kmask[0] & kmask[1] & kmask[2] & kmask[3]) == 0xffffffffu ? 0
                          : ((kmask[1] & kmask[2] & kmask[3]) == 0xffffffffu ? 1
                          : ((kmask[0] & kmask[1] & kmask[2]) == 0xffffffffu ? 2 : 3));

    // ---- multiplier state that no tile changes ----
    // goffv[s]: byte offset, inside a staged tile, of the window row this lane reads in step s
    // (group 2s + h = (ci, ky)); wreg: every weight fragment of the workgroup's channels, so
    // that the K loop reads only input fragments from LDS (filled after the first barrier).
    uint32_t goffv[SU];
    Frag wreg[SU][CB];
#pragma unroll
    for (int s = 0; s < SU; ++s) {
        const int g = min(2 * s + h, p.G - 1);
        const int ci = (int)fdiv((uint32_t)g, p.div_kh);
        goffv[s] = (uint32_t)ci * chb + (uint32_t)(g - ci * p.kh) * rowb;
    }

    // ---- multiplier work for one tile: K loop out of input buffer `buf`, results to `outl` ----
    auto multiply = [&](const Geom &T, uint32_t buf, uint32_t *outl) {
        uint32_t pbase[PXW], shift[PXW];
#pragma unroll
        for (int pb = 0; pb < PXW; ++pb) {
            int oyl, ox;                                  // output row inside the staged tile, column
            if constexpr (POOL) {
                // two whole rows; pixels past them repeat the last one (never pooled)
                const int idx = min((cwave * PXW + pb) * 32 + c32, 2 * p.OW - 1);
                oyl = idx >= p.OW ? 1 : 0;
                ox = idx - oyl * p.OW;
            } else {
                const int m = T.m0 + (cwave * PXW + pb) * 32 + c32;
                const int mm = min(m, ohw - 1);
                const int oy = (int)fdiv((uint32_t)mm, p.div_ow);
                ox = mm - oy * p.OW;
                oyl = oy - T.oyA;
            }
            const int cs = p.padl - p.pw + ox * p.sw - p.front;
            pbase[pb] = (uint32_t)(((oyl * p.sh) * p.pitch + (cs & ~1)) * 2) + 32u + buf * xstride;
            shift[pb] = (uint32_t)(cs & 1) * 16u;
        }
        floatx16 acc[CB][PXW];
        auto kloop = [&](auto mm_tag) {
            constexpr int MM = decltype(mm_tag)::value;
            constexpr int NR = ALIGNED ? 4 : 5;
            // raw dwords of step s; masks and the odd-column shift are applied right before
            // the step's MFMAs, so nothing waits for a read that has just been issued
            auto load_b = [&](int s, uint32_t (&raw)[PXW][NR]) {
#pragma unroll
                for (int pb = 0; pb < PXW; ++pb) {
                    const uint32_t *src = reinterpret_cast<const uint32_t *>(xz + pbase[pb] + goffv[s]);
#pragma unroll
                    for (int q = 0; q < NR; ++q) raw[pb][q] = src[q];
                }
            };
            auto fix_b = [&](int s, const uint32_t (&raw)[PXW][NR], Frag (&b)[PXW]) {
#pragma unroll
                for (int pb = 0; pb < PXW; ++pb) {
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        b[pb].d[q] = ALIGNED ? raw[pb][q]
                                             : __builtin_amdgcn_alignbit(raw[pb][NR - 4 + q], raw[pb][q], shift[pb]);
                    if (MM == 1 || MM == 3) b[pb].d[0] &= kmask[0];
                    if (MM == 3) { b[pb].d[1] &= kmask[1]; b[pb].d[2] &= kmask[2]; }
                    if (MM == 2 || MM == 3) b[pb].d[3] &= kmask[3];
                    if (s >= SU - 2) {              // the only steps that can lie past the last group
                        const bool live = 2 * s + h < p.G;
#pragma unroll
                        for (int q = 0; q < 4; ++q) b[pb].d[q] = live ? b[pb].d[q] : 0u;
                    }
                }
            };
            // Exactly SU steps with no branch between them (steps past the last group multiply
            // zeros), so the LDS reads in flight can be counted.  Step s issues the reads of
            // step s+2, prepares the fragments of step s+1 (read two steps ago) and multiplies
            // those of step s; the group barriers spread the reads and the vector arithmetic
            // between the four MFMAs, which each keep the matrix pipe busy for 32 cycles.
            uint32_t raw[3][PXW][NR];
            Frag bb[2][PXW];
            floatx16 zero;
#pragma unroll
            for (int r = 0; r < 16; ++r) zero[r] = 0.0f;
            load_b(0, raw[0]);
            if (SU > 1) load_b(1, raw[1]);
            fix_b(0, raw[0], bb[0]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < SU; ++s) {
                if (s + 2 < SU) load_b(s + 2, raw[(s + 2) % 3]);
                if (s + 1 < SU) fix_b(s + 1, raw[(s + 1) % 3], bb[(s + 1) & 1]);
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int pb = 0; pb < PXW; ++pb)
                        acc[cb][pb] = mfma16(wreg[s][cb], bb[s & 1][pb], s == 0 ? zero : acc[cb][pb]);
                // MFMA | address arithmetic + reads | MFMA | reads | MFMA | fragment fix-up | MFMA...
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, PXW * (ALIGNED ? 1 : 2), 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, PXW * (ALIGNED ? 1 : 2), 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x002, 32, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, CB * PXW, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        if (mask_mode == 0) kloop(std::integral_constant<int, 0>{});
        else if (mask_mode == 1) kloop(std::integral_constant<int, 1>{});
        else if (mask_mode == 2) kloop(std::integral_constant<int, 2>{});
        else kloop(std::integral_constant<int, 3>{});
        tile_to_lds<CB, PXW, NWC>(acc, outl, cwave, lane, p.relu != 0);
    };

    // ---- common prologue: weights global -> LDS -> fragment layout ----
    weights_park();
    __syncthreads();
    weights_frag();

    if (!mover) {
        // ---- multiplying wavefronts: barrier b ends "tile b-1 multiplied, tile b staged" ----
        __syncthreads();
#pragma unroll
        for (int s = 0; s < SU; ++s)
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const uint4 v = wl[cb * p.G2 * 32 + min(s, p.S - 1) * 64 + lane];
                wreg[s][cb].u = (s < p.S) ? v : make_uint4(0, 0, 0, 0);
            }
        for (int i = 0; i < K; ++i) {
            multiply(geom(i), (uint32_t)(i & 1), reinterpret_cast<uint32_t *>(outl0 + (i & 1) * ostride));
            __syncthreads();
        }
        return;
    }

    // ---- data-moving wavefronts ----
    // Loading wavefronts, per iteration: write the input of tile i+1 (requested an iteration ago)
    // to its buffer, request tile i+2.  Storing wavefronts: write the results of tile i-1 to
    // global memory.  The two kinds have separate memory counters, so a wait for loaded data
    // never also waits for stores; the storing wavefronts never wait for memory at all.
    if (loader) {
        commit_loads(xz + 32);                    // tile 0, requested before the weights
        issue_loads(geom(1));
        __syncthreads();
        commit_loads(xz + 32 + xstride);          // K == 1: a second copy of tile 0, never read
        issue_loads(geom(2));
        __syncthreads();
        for (int i = 1; i < K; ++i) {
            commit_loads(xz + 32 + ((i + 1) & 1) * xstride);
            issue_loads(geom(i + 2));             // clamped to the last tile
            __syncthreads();
        }
        return;
    }
    __syncthreads();
    __syncthreads();
    if constexpr (POOL) {
        for (int i = 1; i < K; ++i) {
            pool_tile_ws(i - 1);
            __syncthreads();
        }
        pool_tile_ws(K - 1);
    } else if (UNAL && (ohw & 7) != 0) {
        for (int i = 1; i < K; ++i) {
            store_tile_ws_grid(i - 1);
            __syncthreads();
        }
        store_tile_ws_grid(K - 1);
    } else {
        for (int i = 1; i < K; ++i) {
            store_tile_ws(i - 1);
            __syncthreads();
        }
        store_tile_ws(K - 1);
    }
}

// ---------------------------------------------------------------------------
// channel-block variant
// LDS: [ weights: S*CB*64 x 16 B ][ input: nchi*RHa*pitch x 16 B ][ output staging ]
// MFMA step s = (chi', tap): lanes 0-31 take channel group chi', lanes 32-63
// take chi' + nchi/2, so the per-step LDS offset is the same for every lane.
// ---------------------------------------------------------------------------

// LDS bank spreading for the staging writes (the XOR layout of Section IV-B).  Input: inside
// every aligned run of 8 staged columns the position is XORed with the run's index (a staging
// thread writes one run of 8 pixels, its neighbours the adjacent runs 128 bytes apart).
// Weights: a fragment's channel slot is XORed with its channel-group index (neighbouring
// staging threads hold different channel groups of the same output channel, whose fragments
// lie a multiple of 1 KB apart).  The K loop applies the same maps when it reads.
// (columns of the last, partial run of a row keep their place: `lim` = pitch rounded down to 8)
__device__ __forceinline__ int xsw(int col, int lim) { return col < lim ? col ^ ((col >> 3) & 7) : col; }
__device__ __forceinline__ int wsw(int cc, int chi) { return cc ^ (chi & 7); }

// weights, 8 channels x T taps per unit, read as T 16-byte loads and transposed
// in registers to T fragments of 8 channels (needs Cin % 8 == 0)
template <int T>
__device__ __forceinline__ void stage_weights_chblock_vec(const ConvParams &p, const uint16_t *__restrict__ w,
                                                          uint4 *wl, int co_base, int CB, int chi0, int t0, int nthr)
{
    const int half_nchi = p.nchi >> 1;
    const int units = CB * 32 * p.nchi;
    // batches of WB units: every load of a batch is issued before the first use
    constexpr int WB = (T >= 16) ? 1 : (T >= 8) ? 4 : 8;     // 4T registers per unit
    for (int u0 = t0; u0 < units; u0 += nthr * WB) {
        uint32_t src[WB][4 * T];
#pragma unroll
        for (int k = 0; k < WB; ++k) {
            const int u = min(u0 + nthr * k, units - 1);
            const int col = (int)fdiv((uint32_t)u, p.div_nchi);
            const int chi = u - col * p.nchi;
            const int co = co_base + col;
            const bool ok = (co < p.Cout) && ((chi0 + chi) * 8 + 8 <= p.Cin);
            // branch-free load (a padding unit re-reads unit 0 and is zeroed)
            const uint4 *g =
                reinterpret_cast<const uint4 *>(w + (ok ? ((size_t)co * p.Cin + (chi0 + chi) * 8) * T : 0));
#pragma unroll
            for (int i = 0; i < T; ++i) {
                const uint4 v = g[i];
                src[k][4 * i + 0] = ok ? v.x : 0u; src[k][4 * i + 1] = ok ? v.y : 0u;
                src[k][4 * i + 2] = ok ? v.z : 0u; src[k][4 * i + 3] = ok ? v.w : 0u;
            }
        }
#pragma unroll
        for (int k = 0; k < WB; ++k) {
            const int u = u0 + nthr * k;
            if (u >= units) break;
            const int col = (int)fdiv((uint32_t)u, p.div_nchi);
            const int chi = u - col * p.nchi;
            const int hh = chi >= half_nchi ? 1 : 0;
            const int chip = chi - hh * half_nchi;
            const int cb = col >> 5, cc = col & 31;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                uint32_t d[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int e0 = (2 * q) * T + t, e1 = (2 * q + 1) * T + t;   // halves (c=2q,t), (c=2q+1,t)
                    const uint32_t sel =
                        ((e0 & 1) ? 0x00000302u : 0x00000100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
                    d[q] = __builtin_amdgcn_perm(src[k][e1 >> 1], src[k][e0 >> 1], sel);
                }
                const int s = chip * T + t;
                wl[((s * CB + cb) * 2 + hh) * 32 + wsw(cc, chi)] = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
    }
}

__device__ __forceinline__ void stage_weights_chblock_scalar(const ConvParams &p, const uint16_t *__restrict__ w,
                                                             uint4 *wl, int co_base, int CB, int chi0, int t0,
                                                             int nthr)
{
    const int T = p.kh * p.kw;
    const int half_nchi = p.nchi >> 1;
    const int units = CB * 32 * p.nchi * T;          // one 16-byte fragment each
    for (int u = t0; u < units; u += nthr) {
        const int t = u % T;
        const int r = u / T;
        const int chi = r % p.nchi;
        const int col = r / p.nchi;
        const int co = co_base + col;
        uint32_t d[4] = {0, 0, 0, 0};
        if (co < p.Cout) {
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                const int ci = (chi0 + chi) * 8 + c;
                if (ci < p.Cin) d[c >> 1] |= (uint32_t)w[((size_t)co * p.Cin + ci) * T + t] << (16 * (c & 1));
            }
        }
        const int hh = chi >= half_nchi ? 1 : 0;
        const int chip = chi - hh * half_nchi;
        const int s = chip * T + t;
        wl[((s * CB + (col >> 5)) * 2 + hh) * 32 + wsw(col & 31, chi)] = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// chi0: first channel group of the pass (the groups of a pass are numbered from 0 in LDS).
// WIDE adds the vector path for 5x5 windows (100 registers per unit: only the multi-pass
// kernel takes it; in the single-pass kernel it would cost the second wavefront per SIMD).
template <bool WIDE = false>
__device__ __forceinline__ void stage_weights_chblock(const ConvParams &p, const uint16_t *__restrict__ w,
                                                      uint4 *wl, int co_base, int CB, int chi0, int t0, int nthr)
{
    const int T = p.kh * p.kw;
    if (T == 9 && (p.Cin & 7) == 0) stage_weights_chblock_vec<9>(p, w, wl, co_base, CB, chi0, t0, nthr);
    else if (T == 1 && (p.Cin & 7) == 0) stage_weights_chblock_vec<1>(p, w, wl, co_base, CB, chi0, t0, nthr);
    else if (WIDE && T == 25 && (p.Cin & 7) == 0) stage_weights_chblock_vec<25>(p, w, wl, co_base, CB, chi0, t0, nthr);
    else stage_weights_chblock_scalar(p, w, wl, co_base, CB, chi0, t0, nthr);
}

// input rows [yA, yA+RH) of image n as [ci/8][row][col][8 channels], channel groups chi0 .. chi0 + nchi - 1
__device__ __forceinline__ void stage_input_chblock(const ConvParams &p, const uint16_t *__restrict__ x, uint4 *xl,
                                                    int n, int yA, int RH, int chi0, int t0, int nthr)
{
    // zero the padding columns of the staged rows
    const int npad = p.pitch - p.W;
    for (int u = t0; u < p.nchi * p.RHa * npad; u += nthr) {
        const int rowi = u / npad;
        const int c = u - rowi * npad;
        const int col = c < p.padl ? c : p.W + c;
        xl[rowi * p.pitch + xsw(col, p.pitch & ~7)] = make_uint4(0, 0, 0, 0);
    }
    if ((p.W & 7) == 0) {
        // 8 channels x 8 pixels per unit, transposed in registers
        const int W8 = p.W >> 3;
        const int nu = p.nchi * p.RHa * W8;
        const size_t chstride = (size_t)p.H * p.W;
        // batches of XB units: every load of a batch is issued before the first use
        constexpr int XB = 3;
        for (int u0 = t0; u0 < nu; u0 += nthr * XB) {
            uint32_t v[XB][8][4];
#pragma unroll
            for (int k = 0; k < XB; ++k) {
                const int u = min(u0 + nthr * k, nu - 1);
                const int q = (int)fdiv((uint32_t)u, p.div_w8);
                const int x8 = u - q * W8;
                const int chi = (int)fdiv((uint32_t)q, p.div_rha);
                const int r = q - chi * p.RHa;
                const int gy = yA + r;
                const bool rowok = r < RH && gy >= 0 && gy < p.H;
                const int ch0 = (chi0 + chi) * 8;
                const uint16_t *src = x + (((size_t)n * p.Cin + ch0) * p.H + (rowok ? gy : 0)) * p.W + 8 * x8;
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const bool ok = rowok && (ch0 + c < p.Cin);
                    // branch-free: a padding channel or row re-reads the tensor's first bytes and is zeroed
                    const uint4 t4 = *reinterpret_cast<const uint4 *>(ok ? src + c * chstride : x);
                    v[k][c][0] = ok ? t4.x : 0u; v[k][c][1] = ok ? t4.y : 0u;
                    v[k][c][2] = ok ? t4.z : 0u; v[k][c][3] = ok ? t4.w : 0u;
                }
            }
#pragma unroll
            for (int k = 0; k < XB; ++k) {
                const int u = u0 + nthr * k;
                if (u >= nu) break;
                const int q = (int)fdiv((uint32_t)u, p.div_w8);
                const int x8 = u - q * W8;
                const int chi = (int)fdiv((uint32_t)q, p.div_rha);
                const int r = q - chi * p.RHa;
                uint4 *dst = xl + (chi * p.RHa + r) * p.pitch;
                const int col0 = p.padl + 8 * x8;
#pragma unroll
                for (int px = 0; px < 8; ++px) {
                    const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
                    uint32_t d[4];
#pragma unroll
                    for (int qq = 0; qq < 4; ++qq)
                        d[qq] = __builtin_amdgcn_perm(v[k][2 * qq + 1][px >> 1], v[k][2 * qq][px >> 1], sel);
                    dst[xsw(col0 + px, p.pitch & ~7)] = make_uint4(d[0], d[1], d[2], d[3]);
                }
            }
        }
    } else {
        const int nu = p.nchi * p.RHa * p.W;
        for (int u = t0; u < nu; u += nthr) {
            const int q = u / p.W;
            const int xg = u - q * p.W;
            const int chi = q / p.RHa;
            const int r = q - chi * p.RHa;
            if (r >= RH) continue;
            const int gy = yA + r;
            uint32_t d[4] = {0, 0, 0, 0};
            if (gy >= 0 && gy < p.H) {
#pragma unroll
                for (int c = 0; c < 8; ++c) {
                    const int ch = (chi0 + chi) * 8 + c;
                    if (ch < p.Cin)
                        d[c >> 1] |= (uint32_t)x[(((size_t)n * p.Cin + ch) * p.H + gy) * p.W + xg] << (16 * (c & 1));
                }
            }
            xl[(chi * p.RHa + r) * p.pitch + xsw(p.padl + xg, p.pitch & ~7)] = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
}

// RES: residual layer (a separate instance, so that the plain one carries no test for it)
template <int CB, int PXW, bool RES>
__global__ __launch_bounds__(256) void merit_conv2d_chblock(ConvParams p, const uint16_t *__restrict__ x,
                                                           const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ res,
                                                           uint16_t *__restrict__ y)
{
    touch_kernarg_lines();
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *wl = reinterpret_cast<uint4 *>(smem);
    uint4 *xl = reinterpret_cast<uint4 *>(smem + p.lds_w_bytes);
    uint32_t *outl = reinterpret_cast<uint32_t *>(smem + p.lds_o_offset);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, h = lane >> 5, c32 = lane & 31;
    const int co_base = blockIdx.y * CB * 32;
    const int ohw = p.OH * p.OW;
    const int half_nchi = p.nchi >> 1;

    const int ntiles = p.N * p.tiles_per_image;
    bool first = true;
    // consecutive tiles share their halo rows: a contiguous run of each round of tiles per XCD
    const int lwg = (int)xcd_band_item(blockIdx.x, (int)(gridDim.x >> 3), (int)(gridDim.x & 7));
    for (int tile = lwg; tile < ntiles; tile += gridDim.x) {
        const int n = (int)fdiv((uint32_t)tile, p.div_tiles);
        const int m0 = (tile - n * p.tiles_per_image) * p.TM;
        const int oyA = (int)fdiv((uint32_t)m0, p.div_ow);
        const int mlast = min(m0 + p.TM, ohw) - 1;
        const int oyB = (int)fdiv((uint32_t)mlast, p.div_ow);
        const int yA = oyA * p.sh - p.ph;
        const int RH = (oyB - oyA) * p.sh + (p.kh - 1) * p.dh + 1;

        __syncthreads();
        if (first) {
            // first tile: half of the wavefronts fetch the weights (once per workgroup) while
            // the other half fetches the input, so the two global-memory round trips overlap
            if (wave < 2) stage_weights_chblock(p, w, wl, co_base, CB, 0, tid, 128);
            else stage_input_chblock(p, x, xl, n, yA, RH, 0, tid - 128, 128);
            first = false;
        } else {
            stage_input_chblock(p, x, xl, n, yA, RH, 0, tid, 256);
        }
        if (RES) stage_residual<CB, 4 * PXW * 32, 256>(p, outl, res, n, co_base, m0, tid);
        __syncthreads();

        int pbase[PXW], pcol[PXW];                  // staged row offset and column of tap kx = 0
        const int lim8 = p.pitch & ~7;
#pragma unroll
        for (int pb = 0; pb < PXW; ++pb) {
            const int m = m0 + (wave * PXW + pb) * 32 + c32;
            const int mm = min(m, ohw - 1);
            const int oy = (int)fdiv((uint32_t)mm, p.div_ow);
            const int ox = mm - oy * p.OW;
            pbase[pb] = ((h * half_nchi * p.RHa) + (oy - oyA) * p.sh) * p.pitch;
            pcol[pb] = (p.padl - p.pw) + ox * p.sw;
        }

        floatx16 acc[CB][PXW];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;

        // K loop.  Step s = (chip, ky, kx), kx fastest; a lone wavefront per SIMD issues about one
        // instruction per 4-5 cycles, so what counts is instructions per step (two MFMAs = 64
        // cycles).  3x3 windows get the nine steps of a channel-group pair unrolled: weight
        // fragments at immediate offsets, the three swizzled tap columns computed once per tile.
        if (p.kh == 3 && p.kw == 3) {
            int xc[PXW][3];
#pragma unroll
            for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
                for (int kx = 0; kx < 3; ++kx) xc[pb][kx] = pbase[pb] + xsw(pcol[pb] + kx * p.dw, lim8);
            for (int chip = 0; chip < half_nchi; ++chip) {
                const uint4 *wa = wl + (chip * 9 * CB) * 64 + h * 32 + wsw(c32, chip + h * half_nchi);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky) {
                    const int rowoff = (chip * p.RHa + ky * p.dh) * p.pitch;
#pragma unroll
                    for (int kx = 0; kx < 3; ++kx) {
                        Frag a[CB], b[PXW];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) a[cb].u = wa[((ky * 3 + kx) * CB + cb) * 64];
#pragma unroll
                        for (int pb = 0; pb < PXW; ++pb) b[pb].u = xl[xc[pb][kx] + rowoff];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                            for (int pb = 0; pb < PXW; ++pb) acc[cb][pb] = mfma16(a[cb], b[pb], acc[cb][pb]);
                    }
                }
            }
        } else {
            int s = 0;
            for (int chip = 0; chip < half_nchi; ++chip) {
                const int wslot = h * 32 + wsw(c32, chip + h * half_nchi);
                for (int ky = 0; ky < p.kh; ++ky) {
                    const int rowoff = (chip * p.RHa + ky * p.dh) * p.pitch;
                    for (int kx = 0; kx < p.kw; ++kx, ++s) {
                        Frag a[CB], b[PXW];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) a[cb].u = wl[(s * CB + cb) * 64 + wslot];
#pragma unroll
                        for (int pb = 0; pb < PXW; ++pb)
                            b[pb].u = xl[pbase[pb] + rowoff + xsw(pcol[pb] + kx * p.dw, lim8)];
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                            for (int pb = 0; pb < PXW; ++pb) acc[cb][pb] = mfma16(a[cb], b[pb], acc[cb][pb]);
                    }
                }
            }
        }
        store_tile<CB, PXW, 4, false>(p, acc, outl, y, n, co_base, m0, tid, RES);
    }
}

// ---- staging of the multi-pass kernel, split into "issue the loads" and "transpose and write
// to LDS", so that the loads of a pass fly while the previous pass is multiplied.  For layers
// the vector staging takes (Cin % 8 == 0, W % 8 == 0, T = 9 or 1 taps); the plan keeps a pass
// within one (T = 9) or two (T = 1) weight units and CP_XU input units per thread: the
// registers that hold a pass in flight must not push the kernel into spilling (a reload from
// scratch waits for every load issued before it, the prefetched ones included).
// weight units (8 channels x T taps of one output channel, 4T registers) per thread
template <int T> struct CpWu { static constexpr int n = T >= 8 ? 1 : 2; };
constexpr int CP_XU = 1;      // input units (8 channels x 8 pixels of one row, 32 registers) per thread

template <int T>
__device__ __forceinline__ void chpipe_issue_w(const ConvParams &p, const uint16_t *__restrict__ w, int co_base,
                                               int CB, int chi0, int tid, uint32_t (&r)[CpWu<T>::n][4 * T])
{
    const int units = CB * 32 * p.nchi;
#pragma unroll
    for (int k = 0; k < CpWu<T>::n; ++k) {
        const int u = min(tid + 256 * k, units - 1);
        const int col = (int)fdiv((uint32_t)u, p.div_nchi);
        const int chi = u - col * p.nchi;
        const int co = co_base + col;
        const bool ok = (co < p.Cout) && ((chi0 + chi) * 8 + 8 <= p.Cin);
        // branch-free load (a padding unit re-reads unit 0 and is zeroed)
        const uint4 *g = reinterpret_cast<const uint4 *>(w + (ok ? ((size_t)co * p.Cin + (chi0 + chi) * 8) * T : 0));
#pragma unroll
        for (int i = 0; i < T; ++i) {
            const uint4 v = g[i];
            r[k][4 * i + 0] = ok ? v.x : 0u; r[k][4 * i + 1] = ok ? v.y : 0u;
            r[k][4 * i + 2] = ok ? v.z : 0u; r[k][4 * i + 3] = ok ? v.w : 0u;
        }
    }
}

template <int T>
__device__ __forceinline__ void chpipe_commit_w(const ConvParams &p, uint4 *wl, int CB, int tid,
                                                const uint32_t (&r)[CpWu<T>::n][4 * T])
{
    const int half_nchi = p.nchi >> 1;
    const int units = CB * 32 * p.nchi;
#pragma unroll
    for (int k = 0; k < CpWu<T>::n; ++k) {
        const int u = tid + 256 * k;
        if (u >= units) break;
        const int col = (int)fdiv((uint32_t)u, p.div_nchi);
        const int chi = u - col * p.nchi;
        const int hh = chi >= half_nchi ? 1 : 0;
        const int chip = chi - hh * half_nchi;
        const int cb = col >> 5, cc = col & 31;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            uint32_t d[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e0 = (2 * q) * T + t, e1 = (2 * q + 1) * T + t;   // halves (c=2q,t), (c=2q+1,t)
                const uint32_t sel =
                    ((e0 & 1) ? 0x00000302u : 0x00000100u) | ((e1 & 1) ? 0x07060000u : 0x05040000u);
                d[q] = __builtin_amdgcn_perm(r[k][e1 >> 1], r[k][e0 >> 1], sel);
            }
            const int s = chip * T + t;
            wl[((s * CB + cb) * 2 + hh) * 32 + wsw(cc, chi)] = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
}

__device__ __forceinline__ void chpipe_issue_x(const ConvParams &p, const uint16_t *__restrict__ x, int n, int yA,
                                               int RH, int chi0, int tid, uint32_t (&v)[CP_XU][8][4])
{
    const int W8 = p.W >> 3;
    const int nu = p.nchi * p.RHa * W8;
    const size_t chstride = (size_t)p.H * p.W;
#pragma unroll
    for (int k = 0; k < CP_XU; ++k) {
        const int u = min(tid + 256 * k, nu - 1);
        const int q = (int)fdiv((uint32_t)u, p.div_w8);
        const int x8 = u - q * W8;
        const int chi = (int)fdiv((uint32_t)q, p.div_rha);
        const int r = q - chi * p.RHa;
        const int gy = yA + r;
        const bool rowok = r < RH && gy >= 0 && gy < p.H;
        const int ch0 = (chi0 + chi) * 8;
        const uint16_t *src = x + (((size_t)n * p.Cin + ch0) * p.H + (rowok ? gy : 0)) * p.W + 8 * x8;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const bool ok = rowok && (ch0 + c < p.Cin);
            // branch-free: a padding channel or row re-reads the tensor's first bytes and is zeroed
            const uint4 t4 = *reinterpret_cast<const uint4 *>(ok ? src + c * chstride : x);
            v[k][c][0] = ok ? t4.x : 0u; v[k][c][1] = ok ? t4.y : 0u;
            v[k][c][2] = ok ? t4.z : 0u; v[k][c][3] = ok ? t4.w : 0u;
        }
    }
}

__device__ __forceinline__ void chpipe_commit_x(const ConvParams &p, uint4 *xl, int tid,
                                                const uint32_t (&v)[CP_XU][8][4])
{
    const int W8 = p.W >> 3;
    const int nu = p.nchi * p.RHa * W8;
#pragma unroll
    for (int k = 0; k < CP_XU; ++k) {
        const int u = tid + 256 * k;
        if (u >= nu) break;
        const int q = (int)fdiv((uint32_t)u, p.div_w8);
        const int x8 = u - q * W8;
        const int chi = (int)fdiv((uint32_t)q, p.div_rha);
        const int r = q - chi * p.RHa;
        uint4 *dst = xl + (chi * p.RHa + r) * p.pitch;
        const int col0 = p.padl + 8 * x8;
#pragma unroll
        for (int px = 0; px < 8; ++px) {
            const uint32_t sel = (px & 1) ? 0x07060302u : 0x05040100u;
            uint32_t d[4];
#pragma unroll
            for (int qq = 0; qq < 4; ++qq)
                d[qq] = __builtin_amdgcn_perm(v[k][2 * qq + 1][px >> 1], v[k][2 * qq][px >> 1], sel);
            dst[xsw(col0 + px, p.pitch & ~7)] = make_uint4(d[0], d[1], d[2], d[3]);
        }
    }
}

// zero the padding columns of the staged rows (they are the same in every pass of a tile)
__device__ __forceinline__ void chpipe_zero_pad(const ConvParams &p, uint4 *xl, int tid)
{
    const int npad = p.pitch - p.W;
    for (int u = tid; u < p.nchi * p.RHa * npad; u += 256) {
        const int rowi = u / npad;
        const int c = u - rowi * npad;
        const int col = c < p.padl ? c : p.W + c;
        xl[rowi * p.pitch + xsw(col, p.pitch & ~7)] = make_uint4(0, 0, 0, 0);
    }
}

// The same for widths that are not a multiple of 8: a unit is one pixel x 8 channels, eight
// 2-byte loads (a lane a pixel, so each of the eight is coalesced along the row).
constexpr int CP_XS = 3;      // such units per thread

__device__ __forceinline__ void chpipe_issue_xs(const ConvParams &p, const uint16_t *__restrict__ x, int n, int yA,
                                                int RH, int chi0, int tid, uint16_t (&v)[CP_XS][8])
{
    const int nu = p.nchi * p.RHa * p.W;
#pragma unroll
    for (int k = 0; k < CP_XS; ++k) {
        const int u = min(tid + 256 * k, nu - 1);
        const int q = (int)fdiv((uint32_t)u, p.div_w);
        const int xg = u - q * p.W;
        const int chi = (int)fdiv((uint32_t)q, p.div_rha);
        const int r = q - chi * p.RHa;
        const int gy = yA + r;
        const bool rowok = r < RH && gy >= 0 && gy < p.H;
        const int ch0 = (chi0 + chi) * 8;
        const uint16_t *src = x + (((size_t)n * p.Cin + ch0) * p.H + (rowok ? gy : 0)) * p.W + xg;
        const size_t chstride = (size_t)p.H * p.W;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const bool ok = rowok && (ch0 + c < p.Cin);
            const uint16_t t = *(ok ? src + c * chstride : x);        // branch-free; zeroed below
            v[k][c] = ok ? t : (uint16_t)0;
        }
    }
}

__device__ __forceinline__ void chpipe_commit_xs(const ConvParams &p, uint4 *xl, int tid,
                                                 const uint16_t (&v)[CP_XS][8])
{
    const int nu = p.nchi * p.RHa * p.W;
#pragma unroll
    for (int k = 0; k < CP_XS; ++k) {
        const int u = tid + 256 * k;
        if (u >= nu) break;
        const int q = (int)fdiv((uint32_t)u, p.div_w);
        const int xg = u - q * p.W;
        uint32_t d[4];
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) d[qq] = (uint32_t)v[k][2 * qq] | ((uint32_t)v[k][2 * qq + 1] << 16);
        xl[q * p.pitch + xsw(p.padl + xg, p.pitch & ~7)] = make_uint4(d[0], d[1], d[2], d[3]);
    }
}

// The same tile and K loop for layers whose weights and input rows do not fit LDS at once: the
// channels go through in passes of p.nchi groups of eight and the accumulators stay in
// registers across the passes (a kernel of its own: accumulators that live across the staging
// code cost the single-pass kernel above 10 % of its speed).
// T = 9 or 1: the pipelined vector staging above (p.pipe says so); T = 0: any shape, a pass is
// staged and then multiplied.
// XV: the input rows take the 16-byte staging (W % 8 == 0), else the per-pixel one.
template <int CB, int PXW, bool RES, int T, bool XV = true>
__global__ __launch_bounds__(256, (CB * PXW == 4 ? 1 : 2)) void merit_conv2d_chpass(ConvParams p, const uint16_t *__restrict__ x,
                                                           const uint16_t *__restrict__ w,
                                                           const uint16_t *__restrict__ res,
                                                           uint16_t *__restrict__ y)
{
    touch_kernarg_lines();
    extern __shared__ __align__(16) uint8_t smem[];
    uint4 *wl = reinterpret_cast<uint4 *>(smem);
    uint4 *xl = reinterpret_cast<uint4 *>(smem + p.lds_w_bytes);
    uint32_t *outl = reinterpret_cast<uint32_t *>(smem + p.lds_o_offset);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, h = lane >> 5, c32 = lane & 31;
    const int co_base = blockIdx.y * CB * 32;
    const int ohw = p.OH * p.OW;
    const int half_nchi = p.nchi >> 1;

    const int ntiles = p.N * p.tiles_per_image;
    bool first = true;
    constexpr bool MULTI = true, multi = true;
    // consecutive tiles share their halo rows: a contiguous run of each round of tiles per XCD
    const int lwg = (int)xcd_band_item(blockIdx.x, (int)(gridDim.x >> 3), (int)(gridDim.x & 7));
    for (int tile = lwg; tile < ntiles; tile += gridDim.x) {
        const int n = (int)fdiv((uint32_t)tile, p.div_tiles);
        const int m0 = (tile - n * p.tiles_per_image) * p.TM;
        const int oyA = (int)fdiv((uint32_t)m0, p.div_ow);
        const int mlast = min(m0 + p.TM, ohw) - 1;
        const int oyB = (int)fdiv((uint32_t)mlast, p.div_ow);
        const int yA = oyA * p.sh - p.ph;
        const int RH = (oyB - oyA) * p.sh + (p.kh - 1) * p.dh + 1;

        int pbase[PXW], pcol[PXW];                  // staged row offset and column of tap kx = 0
        const int lim8 = p.pitch & ~7;
#pragma unroll
        for (int pb = 0; pb < PXW; ++pb) {
            const int m = m0 + (wave * PXW + pb) * 32 + c32;
            const int mm = min(m, ohw - 1);
            const int oy = (int)fdiv((uint32_t)mm, p.div_ow);
            const int ox = mm - oy * p.OW;
            pbase[pb] = ((h * half_nchi * p.RHa) + (oy - oyA) * p.sh) * p.pitch;
            pcol[pb] = (p.padl - p.pw) + ox * p.sw;
        }

        floatx16 acc[CB][PXW];
        auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int pb = 0; pb < PXW; ++pb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[cb][pb][r] = 0.0f;
        };
        if (MULTI) clear_acc();

        // Channels go through LDS in passes of p.nchi groups of eight (one pass when everything
        // fits); the accumulators stay in registers across the passes.
        const int npass = MULTI ? p.nchunks : 1;
        constexpr int TT = T > 0 ? T : 1;
        uint32_t wreg[CpWu<TT>::n][4 * TT], xreg[XV ? CP_XU : 1][8][4];
        uint16_t xsreg[XV ? 1 : CP_XS][8];
        if constexpr (T > 0) {
            chpipe_issue_w<TT>(p, w, co_base, CB, 0, tid, wreg);
            if constexpr (XV) chpipe_issue_x(p, x, n, yA, RH, 0, tid, xreg);
            else chpipe_issue_xs(p, x, n, yA, RH, 0, tid, xsreg);
        }
        for (int ck = 0; ck < npass; ++ck) {
            __syncthreads();                           // the previous pass (or tile) has been read
            const int chi0 = ck * p.nchi;
            if constexpr (T > 0) {
                chpipe_commit_w<TT>(p, wl, CB, tid, wreg);
                if constexpr (XV) chpipe_commit_x(p, xl, tid, xreg);
                else chpipe_commit_xs(p, xl, tid, xsreg);
                if (ck == 0) chpipe_zero_pad(p, xl, tid);
                if (ck + 1 < npass) {                  // the next pass's loads fly under this pass's MFMAs
                    chpipe_issue_w<TT>(p, w, co_base, CB, chi0 + p.nchi, tid, wreg);
                    if constexpr (XV) chpipe_issue_x(p, x, n, yA, RH, chi0 + p.nchi, tid, xreg);
                    else chpipe_issue_xs(p, x, n, yA, RH, chi0 + p.nchi, tid, xsreg);
                }
            } else if (multi) {
                // every pass needs its weights: all wavefronts fetch both (the weights are the
                // larger part)
                stage_weights_chblock<true>(p, w, wl, co_base, CB, chi0, tid, 256);
                stage_input_chblock(p, x, xl, n, yA, RH, chi0, tid, 256);
            } else if (first) {
                // half of the wavefronts fetch the weights (once per workgroup) while the other
                // half fetches the input, so the two global-memory round trips overlap
                if (wave < 2) stage_weights_chblock(p, w, wl, co_base, CB, chi0, tid, 128);
                else stage_input_chblock(p, x, xl, n, yA, RH, chi0, tid - 128, 128);
                first = false;
            } else {
                stage_input_chblock(p, x, xl, n, yA, RH, chi0, tid, 256);
            }
            if (RES && ck == 0) stage_residual<CB, 4 * PXW * 32, 256>(p, outl, res, n, co_base, m0, tid);
            __syncthreads();
            if (!MULTI) clear_acc();

            // K loop.  Step s = (chip, ky, kx), kx fastest; a lone wavefront per SIMD issues about one
            // instruction per 4-5 cycles, so what counts is instructions per step (two MFMAs = 64
            // cycles).  3x3 windows get the nine steps of a channel-group pair unrolled: weight
            // fragments at immediate offsets, the three swizzled tap columns computed once per tile.
            if (p.kh == 3 && p.kw == 3) {
                int xc[PXW][3];
    #pragma unroll
                for (int pb = 0; pb < PXW; ++pb)
    #pragma unroll
                    for (int kx = 0; kx < 3; ++kx) xc[pb][kx] = pbase[pb] + xsw(pcol[pb] + kx * p.dw, lim8);
                for (int chip = 0; chip < half_nchi; ++chip) {
                    const uint4 *wa = wl + (chip * 9 * CB) * 64 + h * 32 + wsw(c32, chip + h * half_nchi);
    #pragma unroll
                    for (int ky = 0; ky < 3; ++ky) {
                        const int rowoff = (chip * p.RHa + ky * p.dh) * p.pitch;
    #pragma unroll
                        for (int kx = 0; kx < 3; ++kx) {
                            Frag a[CB], b[PXW];
    #pragma unroll
                            for (int cb = 0; cb < CB; ++cb) a[cb].u = wa[((ky * 3 + kx) * CB + cb) * 64];
    #pragma unroll
                            for (int pb = 0; pb < PXW; ++pb) b[pb].u = xl[xc[pb][kx] + rowoff];
    #pragma unroll
                            for (int cb = 0; cb < CB; ++cb)
    #pragma unroll
                                for (int pb = 0; pb < PXW; ++pb) acc[cb][pb] = mfma16(a[cb], b[pb], acc[cb][pb]);
                        }
                    }
                }
            } else {
                int s = 0;
                for (int chip = 0; chip < half_nchi; ++chip) {
                    const int wslot = h * 32 + wsw(c32, chip + h * half_nchi);
                    for (int ky = 0; ky < p.kh; ++ky) {
                        const int rowoff = (chip * p.RHa + ky * p.dh) * p.pitch;
                        for (int kx = 0; kx < p.kw; ++kx, ++s) {
                            Frag a[CB], b[PXW];
    #pragma unroll
                            for (int cb = 0; cb < CB; ++cb) a[cb].u = wl[(s * CB + cb) * 64 + wslot];
    #pragma unroll
                            for (int pb = 0; pb < PXW; ++pb)
                                b[pb].u = xl[pbase[pb] + rowoff + xsw(pcol[pb] + kx * p.dw, lim8)];
    #pragma unroll
                            for (int cb = 0; cb < CB; ++cb)
    #pragma unroll
                                for (int pb = 0; pb < PXW; ++pb) acc[cb][pb] = mfma16(a[cb], b[pb], acc[cb][pb]);
                        }
                    }
                }
            }
        }
        store_tile<CB, PXW, 4, false>(p, acc, outl, y, n, co_base, m0, tid, RES);
    }
}

// ---------------------------------------------------------------------------
// Last resort for shapes neither MFMA kernel takes (a window or a channel count whose
// operands do not fit the LDS layouts above): the definition itself on the vector ALU, fp16
// products (exact in fp32) accumulated in fp32 in the order (ci, ky, kx), then the PostLoop of
// the other kernels: + residual, clip, one rounding.  A workgroup owns 256 consecutive pixels
// of one image (a lane a pixel) and DIRECT_CO output channels: an input element is loaded and
// converted once for DIRECT_CO multiply-adds, the weights are the same for the whole
// workgroup (uniform addresses).  Workgroup index = (image, channel block, pixel block),
// pixel block fastest.
constexpr int DIRECT_CO = 8;
constexpr int DIRECT_WTAPS = 1024;      // taps of one input channel held in LDS at a time (32 KB)

__global__ __launch_bounds__(256) void merit_conv2d_direct(ConvParams p, const uint16_t *__restrict__ x,
                                                          const uint16_t *__restrict__ w,
                                                          const uint16_t *__restrict__ res,
                                                          uint16_t *__restrict__ y)
{
    const uint32_t ohw = (uint32_t)(p.OH * p.OW);
    const uint32_t pblocks = (ohw + 255u) / 256u;                      // plain divisions: any extent
    const uint32_t q0 = blockIdx.x / pblocks;
    const uint32_t pb = blockIdx.x - q0 * pblocks;
    const uint32_t n = q0 / (uint32_t)p.co_groups;
    const int co0 = (int)(q0 - n * (uint32_t)p.co_groups) * DIRECT_CO;
    const uint32_t m = pb * 256u + threadIdx.x;                        // pixel of the image
    const uint32_t mm = min(m, ohw - 1u);                              // idle lanes repeat the last pixel
    const int oy = (int)(mm / (uint32_t)p.OW);
    const int ox = (int)(mm - (uint32_t)oy * (uint32_t)p.OW);
    const _Float16 *xh = reinterpret_cast<const _Float16 *>(x) + (size_t)n * p.Cin * p.H * p.W;
    const _Float16 *wh = reinterpret_cast<const _Float16 *>(w);
    const int T = p.kh * p.kw;
    const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
    // The weights of the workgroup's DIRECT_CO output channels for one input channel and a chunk
    // of window rows go to LDS as fp32, [tap][channel]: a tap's 8 weights are two 16-byte
    // reads of one address for the whole wavefront instead of 8 two-byte global loads.
    // Output channels past the last one repeat it (computed, not stored).
    __shared__ __align__(16) float wsh[DIRECT_WTAPS * DIRECT_CO];
    const int kyc = max(1, min(p.kh, DIRECT_WTAPS / p.kw));          // window rows per chunk (kw <= 64)
    float acc[DIRECT_CO];
#pragma unroll
    for (int j = 0; j < DIRECT_CO; ++j) acc[j] = 0.0f;
    for (int ci = 0; ci < p.Cin; ++ci) {
        const _Float16 *xc = xh + (size_t)ci * p.H * p.W;
        for (int ky0 = 0; ky0 < p.kh; ky0 += kyc) {
            const int nky = min(kyc, p.kh - ky0);
            __syncthreads();                                         // the previous chunk has been read
            for (int i = (int)threadIdx.x; i < nky * p.kw * DIRECT_CO; i += 256) {
                const int t = i / DIRECT_CO, j = i - t * DIRECT_CO;
                wsh[i] = (float)wh[(min(co0 + j, p.Cout - 1) * p.Cin + ci) * T + ky0 * p.kw + t];
            }
            __syncthreads();
            for (int ky = 0; ky < nky; ++ky) {
                const int iy = iy0 + (ky0 + ky) * p.dh;
                const bool rowok = iy >= 0 && iy < p.H;
                const _Float16 *xr = xc + (rowok ? iy : 0) * p.W;
                const float4 *wt = reinterpret_cast<const float4 *>(wsh + ky * p.kw * DIRECT_CO);
                for (int kx = 0; kx < p.kw; ++kx) {
                    const int ix = ix0 + kx * p.dw;
                    const bool ok = rowok && ix >= 0 && ix < p.W;
                    const float v = ok ? (float)xr[ok ? ix : 0] : 0.0f;   // zero padding
                    const float4 w0 = wt[2 * kx], w1 = wt[2 * kx + 1];
                    acc[0] = fmaf(v, w0.x, acc[0]); acc[1] = fmaf(v, w0.y, acc[1]);
                    acc[2] = fmaf(v, w0.z, acc[2]); acc[3] = fmaf(v, w0.w, acc[3]);
                    acc[4] = fmaf(v, w1.x, acc[4]); acc[5] = fmaf(v, w1.y, acc[5]);
                    acc[6] = fmaf(v, w1.z, acc[6]); acc[7] = fmaf(v, w1.w, acc[7]);
                }
            }
        }
    }
    if (m < ohw) {
#pragma unroll
        for (int j = 0; j < DIRECT_CO; ++j) {
            if (co0 + j >= p.Cout) break;
            const size_t o = ((size_t)n * p.Cout + (co0 + j)) * ohw + m;
            float a = acc[j];
            if (p.residual) a += (float)reinterpret_cast<const _Float16 *>(res)[o];
            if (p.relu) a = fmaxf(a, 0.0f);
            const _Float16 h = (_Float16)a;                           // round to nearest even
            y[o] = __builtin_bit_cast(uint16_t, h);
        }
    }
}

int conv_direct_channels() { return DIRECT_CO; }

// ---------------------------------------------------------------------------
template <typename K>
static hipError_t launch(K kernel, const ConvParams &p, const void *x, const void *w, const void *r, void *y,
                         hipStream_t s, uint32_t gx, size_t lds_bytes, uint32_t nthreads = 256)
{
    // raise this kernel instance's dynamic-LDS limit to the 160 KB a gfx950 workgroup may
    // use; done once per instance (the static lives in this template instantiation)
    static std::atomic<int> raised{0};
    if (hipError_t e = raise_lds_limit_once(reinterpret_cast<const void *>(kernel), raised); e != hipSuccess) return e;
    hipLaunchKernelGGL(kernel, dim3(gx, (uint32_t)p.co_groups), dim3(nthreads), lds_bytes, s, p,
                       reinterpret_cast<const uint16_t *>(x), reinterpret_cast<const uint16_t *>(w),
                       reinterpret_cast<const uint16_t *>(r), reinterpret_cast<uint16_t *>(y));
    return hipGetLastError();
}

size_t conv_lds_bytes(const ConvParams &p)
{
    return (size_t)p.lds_total;
}

// number of compute units of the current device (cached; 256 on MI355X)
int device_cu_count()
{
    static std::atomic<int> cus{0};
    int c = cus.load(std::memory_order_relaxed);
    if (c == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            c = v;
        else
            c = 256;
        cus.store(c, std::memory_order_relaxed);
    }
    return c;
}

hipError_t launch_conv2d(const ConvParams &p, const void *x, const void *w, const void *r, void *y, hipStream_t s)
{
    const int64_t ntiles = (int64_t)p.N * p.tiles_per_image;
    if (ntiles == 0) return hipSuccess;
    if (p.variant == CONV_CHWS) return launch_conv2d_chws(p, x, w, r, y, s, false);
    if (p.variant == CONV_DIRECT) {                // one workgroup per 256 pixels x 8 channels
        hipLaunchKernelGGL(merit_conv2d_direct, dim3((uint32_t)ntiles), dim3(256), 0, s, p,
                           reinterpret_cast<const uint16_t *>(x), reinterpret_cast<const uint16_t *>(w),
                           reinterpret_cast<const uint16_t *>(r), reinterpret_cast<uint16_t *>(y));
        return hipGetLastError();
    }
    // persistent grid: as many workgroups as fit on the chip at once, at most one per tile
    int64_t slots = (int64_t)device_cu_count() * p.wg_per_cu / p.co_groups;
    if (slots < 1) slots = 1;
    const uint32_t gx = (uint32_t)(ntiles < slots ? ntiles : slots);
    const size_t lds = conv_lds_bytes(p);
    if (p.variant == CONV_PLANAR_SMALLC && p.ws) {
#define MERIT_PLANAR_WS(CBv, SUv)                                                                          \
    do {                                                                                                   \
        if (p.pool) {                                                                                      \
            const uint32_t gp = (uint32_t)((int64_t)p.N * p.NB);                                           \
            if (p.aligned) return launch(merit_conv2d_planar_ws<CBv, true, SUv, true>, p, x, w, r, y, s, gp, lds, 512);  \
            return launch(merit_conv2d_planar_ws<CBv, false, SUv, true>, p, x, w, r, y, s, gp, lds, 512);     \
        }                                                                                                  \
        if (p.unal) {                                                                                      \
            if (p.aligned) return launch(merit_conv2d_planar_ws<CBv, true, SUv, false, true>, p, x, w, r, y, s, gx, lds, 512); \
            return launch(merit_conv2d_planar_ws<CBv, false, SUv, false, true>, p, x, w, r, y, s, gx, lds, 512); \
        }                                                                                                  \
        if (p.aligned) return launch(merit_conv2d_planar_ws<CBv, true, SUv, false>, p, x, w, r, y, s, gx, lds, 512); \
        return launch(merit_conv2d_planar_ws<CBv, false, SUv, false>, p, x, w, r, y, s, gx, lds, 512);        \
    } while (0)
        switch (p.CB * 100 + p.su) {
        case 204: MERIT_PLANAR_WS(2, 4);
        case 206: MERIT_PLANAR_WS(2, 6);
        case 208: MERIT_PLANAR_WS(2, 8);
        case 211: MERIT_PLANAR_WS(2, 11);
        case 212: MERIT_PLANAR_WS(2, 12);
        case 104: MERIT_PLANAR_WS(1, 4);
        case 106: MERIT_PLANAR_WS(1, 6);
        case 108: MERIT_PLANAR_WS(1, 8);
        case 111: MERIT_PLANAR_WS(1, 11);
        case 112: MERIT_PLANAR_WS(1, 12);
        default: return hipErrorInvalidValue;
        }
#undef MERIT_PLANAR_WS
    }
    if (p.variant == CONV_PLANAR_SMALLC) {
        // one batch of 5 staging units per thread covers a tile => next-tile prefetch
        const int nt = p.NW * 64;
        const bool pf = (p.W % 8 == 0) && ((int64_t)p.Cin * p.RHa * (p.pitch / 8) <= nt * 5);
#define MERIT_PLANAR(CBv, PXv, NWv)                                                                        \
    do {                                                                                                   \
        if (p.aligned && pf) return launch(merit_conv2d_planar<CBv, PXv, NWv, true, true>, p, x, w, r, y, s, gx, lds, nt);   \
        if (p.aligned) return launch(merit_conv2d_planar<CBv, PXv, NWv, true, false>, p, x, w, r, y, s, gx, lds, nt);        \
        if (pf) return launch(merit_conv2d_planar<CBv, PXv, NWv, false, true>, p, x, w, r, y, s, gx, lds, nt);               \
        return launch(merit_conv2d_planar<CBv, PXv, NWv, false, false>, p, x, w, r, y, s, gx, lds, nt);                      \
    } while (0)
        if (p.NW == 8) {
            if (p.CB == 2) MERIT_PLANAR(2, 1, 8);
            MERIT_PLANAR(1, 1, 8);
        }
        if (p.CB == 2 && p.PXW == 2) MERIT_PLANAR(2, 2, 4);
        if (p.CB == 2 && p.PXW == 1) MERIT_PLANAR(2, 1, 4);
        if (p.CB == 1 && p.PXW == 2) MERIT_PLANAR(1, 2, 4);
        MERIT_PLANAR(1, 1, 4);
#undef MERIT_PLANAR
    }
#define MERIT_CHBLOCK(CBv, PXv)                                                                   \
    do {                                                                                          \
        if (p.nchunks > 1) {                                                                      \
            if (p.pipe == 9 && (p.W & 7) == 0) {                                                  \
                if (p.residual) return launch(merit_conv2d_chpass<CBv, PXv, true, 9>, p, x, w, r, y, s, gx, lds);  \
                return launch(merit_conv2d_chpass<CBv, PXv, false, 9>, p, x, w, r, y, s, gx, lds);   \
            }                                                                                     \
            if (p.pipe == 1 && (p.W & 7) == 0) {                                                  \
                if (p.residual) return launch(merit_conv2d_chpass<CBv, PXv, true, 1>, p, x, w, r, y, s, gx, lds);  \
                return launch(merit_conv2d_chpass<CBv, PXv, false, 1>, p, x, w, r, y, s, gx, lds);   \
            }                                                                                     \
            if (p.pipe == 9) {                                                                    \
                if (p.residual) return launch(merit_conv2d_chpass<CBv, PXv, true, 9, false>, p, x, w, r, y, s, gx, lds);  \
                return launch(merit_conv2d_chpass<CBv, PXv, false, 9, false>, p, x, w, r, y, s, gx, lds);   \
            }                                                                                     \
            if (p.pipe == 1) {                                                                    \
                if (p.residual) return launch(merit_conv2d_chpass<CBv, PXv, true, 1, false>, p, x, w, r, y, s, gx, lds);  \
                return launch(merit_conv2d_chpass<CBv, PXv, false, 1, false>, p, x, w, r, y, s, gx, lds);   \
            }                                                                                     \
            if (p.residual) return launch(merit_conv2d_chpass<CBv, PXv, true, 0>, p, x, w, r, y, s, gx, lds);  \
            return launch(merit_conv2d_chpass<CBv, PXv, false, 0>, p, x, w, r, y, s, gx, lds);    \
        }                                                                                         \
        if (p.residual) return launch(merit_conv2d_chblock<CBv, PXv, true>, p, x, w, r, y, s, gx, lds); \
        return launch(merit_conv2d_chblock<CBv, PXv, false>, p, x, w, r, y, s, gx, lds);          \
    } while (0)
    if (p.CB == 2 && p.PXW == 2) MERIT_CHBLOCK(2, 2);
    if (p.CB == 2 && p.PXW == 1) MERIT_CHBLOCK(2, 1);
    if (p.CB == 1 && p.PXW == 2) MERIT_CHBLOCK(1, 2);
    MERIT_CHBLOCK(1, 1);
#undef MERIT_CHBLOCK
}

const char *conv_kernel_name(const ConvParams &p)
{
    if (p.variant == CONV_PLANAR_SMALLC && p.ws && p.pool) return "merit_conv2d_planar_ws_pool";
    if (p.variant == CONV_PLANAR_SMALLC) return p.ws ? "merit_conv2d_planar_ws" : "merit_conv2d_planar";
    if (p.variant == CONV_DIRECT) return "merit_conv2d_direct";
    if (p.variant == CONV_CHWS) return p.pool ? "merit_conv2d_chws_pool" : "merit_conv2d_chws";
    return p.nchunks > 1 ? "merit_conv2d_chpass" : "merit_conv2d_chblock";
}

}  // namespace merit
