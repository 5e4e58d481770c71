// Host side of the library: plan validation, derived geometry, and the C ABI.
//
// A plan holds the paper's transform descriptor (per index an axis d_j, stride
// s_j and offset o_j per operand; Section III-C, Eq. 5) after it has been
// matched against the three index patterns the kernels implement, plus the
// tile / halo geometry derived from it with the footprint rule of Section
// IV-A, Eq. 9.  No GPU call happens here.
#include <atomic>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <new>

#include "merit_internal.h"

using namespace merit;

namespace merit {
size_t conv_lds_bytes(const ConvParams &p);
}

namespace {

constexpr int64_t LDS_LIMIT = 160 * 1024;       // per workgroup on gfx950
constexpr int64_t INT_LIMIT = 1ll << 30;

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int64_t round_up(int64_t a, int64_t b) { return cdiv(a, b) * b; }

// FastDiv is exact when (nmax + d) * d < 2^32.
inline bool fastdiv_ok(int64_t nmax, int64_t d) { return d >= 1 && (nmax + d) * d < (1ll << 32); }

bool operand_is(const merit_operand &o, int n_index, const int *axis, const int64_t *stride,
                const int64_t *offset /* may hold INT64_MIN = "don't care" */)
{
    for (int j = 0; j < n_index; ++j) {
        if (o.axis[j] != axis[j]) return false;
        if (axis[j] == MERIT_AXIS_UNUSED) continue;
        if (stride && stride[j] != INT64_MIN && o.stride[j] != stride[j]) return false;
        if (offset && offset[j] != INT64_MIN && o.offset[j] != offset[j]) return false;
    }
    return true;
}

int64_t out_extent(int64_t I, int64_t k, int64_t s, int64_t p) { return (I + 2 * p - k) / s + 1; }

// ---------------------------------------------------------------- pooling ---
merit_status derive_pool(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    const bool is_avg = d.op == MERIT_OP_POOL_AVG;
    if (d.dtype != MERIT_F32) return MERIT_ERR_UNSUPPORTED;
    if (d.pad != (is_avg ? MERIT_PAD_EXCLUDE : MERIT_PAD_NEG_INF)) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 4 || d.n_acc != 2) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 4 || d.b.ndim != 0) return MERIT_ERR_UNSUPPORTED;
    const int axis[6] = {0, 1, 2, 3, 2, 3};
    const int64_t DC = INT64_MIN;
    const int64_t stride[6] = {1, 1, DC, DC, 1, 1};
    const int64_t offset[6] = {0, 0, 0, 0, DC, DC};
    if (!operand_is(d.a, 6, axis, stride, offset)) return MERIT_ERR_UNSUPPORTED;

    const int64_t N = d.a.shape[0], C = d.a.shape[1], H = d.a.shape[2], W = d.a.shape[3];
    const int64_t OH = d.range[2], OW = d.range[3], kh = d.range[4], kw = d.range[5];
    const int64_t sh = d.a.stride[2], sw = d.a.stride[3];
    const int64_t ph = -d.a.offset[4], pw = -d.a.offset[5];
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
        return MERIT_ERR_INVALID_ARG;
    if (d.range[0] != N || d.range[1] != C) return MERIT_ERR_SHAPE;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return MERIT_ERR_SHAPE;
    if (OH != out_extent(H, kh, sh, ph) || OW != out_extent(W, kw, sw, pw)) return MERIT_ERR_SHAPE;
    if (N * C >= INT_LIMIT || H * W >= INT_LIMIT || kh > 64 || kw > 64 || sh > 64 || sw > 64)
        return MERIT_ERR_UNSUPPORTED;

    PoolParams &p = pl->pool;
    p.NC = (int)(N * C); p.H = (int)H; p.W = (int)W; p.OH = (int)OH; p.OW = (int)OW;
    p.kh = (int)kh; p.kw = (int)kw; p.sh = (int)sh; p.sw = (int)sw; p.ph = (int)ph; p.pw = (int)pw;
    p.is_avg = is_avg ? 1 : 0;

    // row-strip variants: full-width strips, 16-byte accesses
    int variant = POOL_TILE_GENERIC;
    // staged rows carry 4 fill columns on either side; the last thread of a row reads
    // whole 16-byte chunks up to float 4*C1 past its span start
    const int64_t C1 = (4 - pw + 3 * sw + kw + 3) / 4;
    const bool rows_ok = (W % 4 == 0) && (OW % 4 == 0) && pw <= 4 &&
                         ((OW - 4) * sw + 4 * C1 <= W + 8);
    if (rows_ok) {
        if (kh == 3 && kw == 3 && sh == 2 && sw == 2 && pw == 1) variant = POOL_ROWS_K3S2P1;
        else if (kh == 2 && kw == 2 && sh == 2 && sw == 2 && pw == 0) variant = POOL_ROWS_K2S2P0;
        // (3x3 at stride 1: on request only -- the two-columns-per-lane kernel below is as fast or faster on every
        // size measured: 32 x 64 x 56 x 56 15.4 against 18.0 us, 8 x 64 x 112 x 112 14.7 against 17.8, 32 x 512 x 8 x 8 5.1 against 10.1)
        else if (kh == 3 && kw == 3 && sh == 1 && sw == 1 && pw == 1 && pl->tile_req[2] > 0) variant = POOL_ROWS_K3S1P1;
    }
    // streaming variant: register-resident strips, no LDS (3x3 / stride 2 / pad 1, W <= 256)
    const bool stream_ok = kh == 3 && kw == 3 && sh == 2 && sw == 2 && ph == 1 && pw == 1 &&
                           (W % 4 == 0) && W <= 256 && pl->tile_req[3] <= 0;
    if (stream_ok) {
        int64_t TH = 4;             // measured best on the 112x112 workload (4 < 7 < 8)
        if (pl->tile_req[2] > 0) TH = pl->tile_req[2];
        if (TH == 4 || TH == 7 || TH == 8) {
            int lg_shift = 0;
            while ((1 << lg_shift) < W / 4) ++lg_shift;
            p.variant = variant = POOL_STREAM_K3S2P1;
            p.TH = (int)TH; p.TW = (int)OW;
            p.tiles_y = (int)cdiv(OH, TH); p.tiles_x = 1;
            p.RH = 0; p.RW = 0; p.pitch = 0;
            p.lg_shift = lg_shift;
            const int64_t items = N * C * p.tiles_y;
            if (items >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;
            p.items = (int)items;
            p.grid = (int)cdiv(items, 4 * (64 >> lg_shift));
        }
    }
    if (variant != POOL_TILE_GENERIC && variant != POOL_STREAM_K3S2P1) {
        const int64_t pitch = W + 8;
        // strip height: as many output rows as keep the staged rows within ~16 KB,
        // then balanced so that all strips of a plane are (nearly) equal
        int64_t TH = (16 * 1024 / (pitch * 4) - kh) / sh + 1;
        if (TH < 1) TH = 1;
        if (TH > OH) TH = OH;
        TH = cdiv(OH, cdiv(OH, TH));
        if (pl->tile_req[2] > 0) TH = pl->tile_req[2] < OH ? pl->tile_req[2] : OH;
        const int64_t RH = (TH - 1) * sh + kh;
        if (RH * pitch * 4 > LDS_LIMIT || !fastdiv_ok(RH * (pitch / 4), pitch / 4) ||
            !fastdiv_ok(TH * (OW / 4), OW / 4)) {
            variant = POOL_TILE_GENERIC;
        } else {
            p.variant = variant;
            p.TH = (int)TH; p.TW = (int)OW;
            p.tiles_y = (int)cdiv(OH, TH); p.tiles_x = 1;
            p.RH = (int)RH; p.RW = (int)pitch; p.pitch = (int)pitch;
            p.div_p4 = make_fastdiv((uint32_t)(pitch / 4));
            p.div_ow4 = make_fastdiv((uint32_t)(OW / 4));
        }
    }
    // 3x3 / stride 2 (padding 0 or 1) and 2x2 / stride 2 (no padding) on a width the 16-byte kernels do not
    // take: a lane per two output columns, whose input columns are one 16-byte load (W >= 8), in groups of
    // 4 to 64 lanes; 3x3 on narrower planes: a lane per output column
    // (3x3 at stride 1, the pooling branch of an inception module on 35, 17 and 7 columns: the same kernel, 8 output rows
    // per group, any width of 4 and more)
    const bool k3 = kh == 3 && kw == 3 && ph <= 1 && pw <= 1, k2 = kh == 2 && kw == 2 && ph == 0 && pw == 0 && W >= 8;
    const bool s1 = k3 && sh == 1 && sw == 1 && W >= 4;
    if (variant == POOL_TILE_GENERIC && (((k3 || k2) && sh == 2 && sw == 2) || s1) &&
        !(OH == 1 && OW == 1) && pl->tile_req[2] <= 0 && pl->tile_req[3] <= 0 && H * W < INT_LIMIT) {
        const bool two = W >= 8 || s1;
        const int64_t th = s1 ? 8 : 4;
        const int64_t cols = two ? 128 : 64;                // output columns of a full group of 64 lanes
        int lg_shift = 0;                                   // items per wavefront = 1 << lg_shift
        while (lg_shift < (two ? 4 : 2) && (cols >> (lg_shift + 1)) >= OW) ++lg_shift;
        const int64_t chunks = cdiv(OW, cols), strips = cdiv(OH, th);
        const int64_t items = N * C * chunks * strips;
        // (2x2 windows on small launches stay on the tile kernel: 8 x 512 x 14 x 14 is 128 workgroups here, 6.1 us against 5.5)
        if (items < INT_LIMIT && fastdiv_ok(items, chunks) && fastdiv_ok(items, strips) &&
            (k3 || s1 || cdiv(items, 4 * (1 << lg_shift)) >= 512)) {
            p.variant = variant = two ? POOL_LANES2_K3S2 : POOL_LANES_K3S2;
            p.TH = (int)th; p.TW = (int)(OW < cols ? OW : cols);
            p.tiles_y = (int)strips; p.tiles_x = (int)chunks;
            p.RH = p.RW = p.pitch = 0;
            p.lg_shift = lg_shift;
            p.items = (int)items;
            p.div_tiles_x = make_fastdiv((uint32_t)chunks);
            p.div_tiles_y = make_fastdiv((uint32_t)strips);
            p.grid = (int)cdiv(items, 4 * (1 << lg_shift));
        }
    }
    // one output per plane (global pooling): a wavefront per plane, no staging
    if (variant == POOL_TILE_GENERIC && OH == 1 && OW == 1 && pl->tile_req[2] <= 0 && pl->tile_req[3] <= 0 &&
        H * W < INT_LIMIT) {
        p.variant = variant = POOL_PLANE;
        p.TH = p.TW = 1; p.tiles_y = p.tiles_x = 1;
        p.RH = p.RW = p.pitch = 0;
        // lanes per plane: about four in-range window elements each, 4 to 64
        const int64_t y0 = std::max<int64_t>(-ph, 0), y1 = std::min<int64_t>(-ph + kh, H);
        const int64_t x0 = std::max<int64_t>(-pw, 0), x1 = std::min<int64_t>(-pw + kw, W);
        const int64_t rw = std::max<int64_t>(x1 - x0, 1), cnt = std::max<int64_t>(y1 - y0, 0) * rw;
        int lg = 0;                                         // planes per wavefront = 1 << lg
        while (lg < 4 && (64 >> (lg + 1)) * 4 >= cnt) ++lg;
        p.lg_shift = lg;
        const int64_t g = cdiv((int64_t)p.NC, 4 << lg);
        if (g >= (1ll << 31)) return MERIT_ERR_UNSUPPORTED;
        p.grid = (int)g;
    }
    if (variant == POOL_TILE_GENERIC) {
        p.variant = POOL_TILE_GENERIC;
        int64_t TW = OW < 64 ? OW : 64;
        int64_t TH = OH < 16 ? OH : 16;
        if (pl->tile_req[2] > 0) TH = pl->tile_req[2] < OH ? pl->tile_req[2] : OH;
        if (pl->tile_req[3] > 0) TW = pl->tile_req[3] < OW ? pl->tile_req[3] : OW;
        // shrink until the staged region fits comfortably
        for (;;) {
            const int64_t RH = (TH - 1) * sh + kh, RW = (TW - 1) * sw + kw;
            if (RH * (RW + 1) * 4 <= 64 * 1024 || (TH == 1 && TW == 1)) break;
            if (TH > 1) TH = (TH + 1) / 2; else TW = (TW + 1) / 2;
        }
        const int64_t RH = (TH - 1) * sh + kh, RW = (TW - 1) * sw + kw;
        if (RH * (RW + 1) * 4 > LDS_LIMIT) return MERIT_ERR_UNSUPPORTED;
        if (!fastdiv_ok(RH * RW, RW) || !fastdiv_ok(TH * TW, TW)) return MERIT_ERR_UNSUPPORTED;
        p.TH = (int)TH; p.TW = (int)TW;
        p.tiles_y = (int)cdiv(OH, TH); p.tiles_x = (int)cdiv(OW, TW);
        p.RH = (int)RH; p.RW = (int)RW; p.pitch = (int)RW + 1;
        p.div_rw = make_fastdiv((uint32_t)RW);
        p.div_tw = make_fastdiv((uint32_t)TW);
    }
    if (variant != POOL_STREAM_K3S2P1 && variant != POOL_PLANE && variant != POOL_LANES_K3S2 && variant != POOL_LANES2_K3S2) {
        const int64_t g = (int64_t)p.NC * p.tiles_y * p.tiles_x;
        if (g >= (1ll << 31)) return MERIT_ERR_UNSUPPORTED;
        p.grid = (int)g;
    }
    const int64_t grid = p.grid;

    pl->out_ndim = 4;
    pl->out_shape[0] = N; pl->out_shape[1] = C; pl->out_shape[2] = OH; pl->out_shape[3] = OW;
    merit_launch_info &li = pl->info;
    li.kernel = pool_kernel_name(p);
    li.grid[0] = grid; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = (int64_t)p.RH * p.pitch * 4;
    li.tile[0] = 1; li.tile[1] = 1; li.tile[2] = p.TH; li.tile[3] = p.TW; li.tile[4] = kh; li.tile[5] = kw;
    return MERIT_OK;
}

// ----------------------------------------------------------- block matching ---
merit_status derive_sad(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_U8 || d.pad != MERIT_PAD_CLAMP) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 2 || d.n_acc != 4) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 2 || d.b.ndim != 2) return MERIT_ERR_UNSUPPORTED;
    const int64_t B = d.range[4], n = d.range[2];
    if (B <= 0 || n <= 0 || d.range[5] != B || d.range[3] != n || (n % 2) == 0) return MERIT_ERR_SHAPE;
    const int64_t R = (n - 1) / 2;
    const int axis_ref[6] = {0, 1, 0, 1, 0, 1};
    const int64_t stride_ref[6] = {B, B, 1, 1, 1, 1};
    const int64_t offset_ref[6] = {0, 0, -R, -R, 0, 0};
    const int axis_cur[6] = {0, 1, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 0, 1};
    const int64_t stride_cur[6] = {B, B, 0, 0, 1, 1};
    const int64_t offset_cur[6] = {0, 0, 0, 0, 0, 0};
    if (!operand_is(d.a, 6, axis_ref, stride_ref, offset_ref)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 6, axis_cur, stride_cur, offset_cur)) return MERIT_ERR_UNSUPPORTED;
    const int64_t H = d.a.shape[0], W = d.a.shape[1];
    if (H <= 0 || W <= 0) return MERIT_ERR_INVALID_ARG;
    if (d.b.shape[0] != H || d.b.shape[1] != W) return MERIT_ERR_SHAPE;
    // blocks that reach past the edge (B does not divide H or W) read both frames clamped
    if (d.range[0] != cdiv(H, B) || d.range[1] != cdiv(W, B)) return MERIT_ERR_SHAPE;
    // key packing: SAD < 2^18 and raster index < 2^14 share one u32
    if (B % 4 || B > 32 || R > 63) return MERIT_ERR_UNSUPPORTED;
    if (H * W >= INT_LIMIT || cdiv(H, B) * cdiv(W, B) >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;

    SadParams &p = pl->sad;
    p.H = (int)H; p.W = (int)W; p.B = (int)B; p.R = (int)R; p.n = (int)n;
    p.nby = (int)cdiv(H, B); p.nbx = (int)cdiv(W, B);
    p.win = (int)(B + 2 * R);
    const int64_t cols4 = cdiv(p.win, 4);
    p.pitch = (int)((cols4 + 1) * 4);
    p.variant = SAD_GENERIC;
    p.bpw = 1; p.groups_x = p.nbx;
    if (!fastdiv_ok(n * n, n) || !fastdiv_ok((int64_t)p.win * cols4, cols4)) return MERIT_ERR_UNSUPPORTED;
    p.div_n = make_fastdiv((uint32_t)n);
    p.div_win4 = make_fastdiv((uint32_t)cols4);
    p.div_nbx = make_fastdiv((uint32_t)p.nbx);

    // row-scan kernel: 16x16 blocks, four blocks per workgroup, instances for R = 16 and 32;
    // a tile request of one block per workgroup keeps the generic kernel
    int64_t grid = (int64_t)p.nby * p.nbx;
    int64_t lds = ((int64_t)p.win * (p.pitch / 4) + 1 + B * (B / 4) + 4) * 4;
    int64_t tile_bx = 1;
    // (the row-scan kernels fetch the current block in aligned dwords: W % 4 == 0; any H)
    const bool rowscan_ok = W % 4 == 0;
    if (rowscan_ok && B == 16 && (R == 16 || R == 32) && pl->tile_req[1] != 1) {
        const int64_t c4 = cdiv(4 * 16 + 2 * R, 4);
        if (fastdiv_ok((16 + 2 * R) * c4, c4)) {
            p.variant = SAD_ROWSCAN_B16;
            p.bpw = 4;
            p.groups_x = (int)cdiv(p.nbx, 4);
            p.pitch = (int)((c4 + 1) * 4);
            p.div_win4 = make_fastdiv((uint32_t)c4);
            grid = (int64_t)p.nby * p.groups_x;
            lds = ((16 + 2 * R) * (c4 + 1) + 1) * 4;
            tile_bx = 4;
        }
    }

    // two blocks per wavefront, eight per workgroup: 8x8 blocks with R = 8 or 16, 16x16 blocks
    // with R = 16 (a tile request of four blocks per workgroup keeps the one-block-per-wavefront
    // kernel there)
    if (rowscan_ok && ((B == 8 && (R == 8 || R == 16)) || (B == 16 && R == 16)) && pl->tile_req[1] != 1 &&
        pl->tile_req[1] != 4) {
        const int64_t c4 = cdiv(8 * B + 2 * R, 4);
        if (fastdiv_ok((B + 2 * R) * c4, c4)) {
            p.variant = SAD_ROWSCAN_PAIR;
            p.bpw = 8;
            p.groups_x = (int)cdiv(p.nbx, 8);
            p.pitch = (int)((c4 + 1) * 4);
            p.div_win4 = make_fastdiv((uint32_t)c4);
            grid = (int64_t)p.nby * p.groups_x;
            lds = ((B + 2 * R) * (c4 + 1) + 1) * 4;
            tile_bx = 8;
        }
    }

    p.xq = (int)(grid / 8); p.xr = (int)(grid % 8);
    pl->out_ndim = 2;
    pl->out_shape[0] = p.nby; pl->out_shape[1] = p.nbx;
    merit_launch_info &li = pl->info;
    li.kernel = sad_kernel_name(p);
    li.grid[0] = grid; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = lds;
    li.tile[0] = 1; li.tile[1] = tile_bx; li.tile[2] = n; li.tile[3] = n; li.tile[4] = B; li.tile[5] = B;
    return MERIT_OK;
}

// -------------------------------------------------------- separable filter ---
merit_status derive_sep(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_F32 || d.pad != MERIT_PAD_CLAMP) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 3 || d.n_acc != 2) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 3 || d.b.ndim != 1) return MERIT_ERR_UNSUPPORTED;
    const int64_t N = d.a.shape[0], H = d.a.shape[1], W = d.a.shape[2], k = d.b.shape[0];
    if (N < 0 || H <= 0 || W <= 0 || k <= 0) return MERIT_ERR_INVALID_ARG;
    const int64_t c = k / 2;
    const int axis_x[5] = {0, 1, 2, 1, 2};
    const int64_t stride_x[5] = {1, 1, 1, 1, 1};
    const int64_t offset_x[5] = {0, 0, 0, -c, -c};
    const int axis_k[5] = {MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 0};
    const int64_t stride_k[5] = {0, 0, 0, 0, 1};
    const int64_t offset_k[5] = {0, 0, 0, 0, 0};
    if (!operand_is(d.a, 5, axis_x, stride_x, offset_x)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 5, axis_k, stride_k, offset_k)) return MERIT_ERR_UNSUPPORTED;
    if (d.range[0] != N || d.range[1] != H || d.range[2] != W || d.range[3] != k || d.range[4] != k)
        return MERIT_ERR_SHAPE;
    if (k > 32 || H * W >= INT_LIMIT || N * H * W >= (1ll << 40)) return MERIT_ERR_UNSUPPORTED;

    SepParams &p = pl->sep;
    p.N = (int)N; p.H = (int)H; p.W = (int)W; p.k = (int)k; p.c = (int)c;
    p.c4 = (int)round_up(c, 4);
    // staged rows RH = TH + k - 1: about 64, more for long windows (whose halo rows the row pass
    // also computes); TH a multiple of 4 (the column pass works on 4 x 4 patches)
    int64_t rows = k <= 16 ? 64 : 96;                     // the kernel keeps rows / 32 row-pass units per thread
    if (pl->tile_req[1] > 0) {                            // staged rows per workgroup, at most
        if (pl->tile_req[1] < k + 3 || pl->tile_req[1] > rows) return MERIT_ERR_UNSUPPORTED;
        rows = pl->tile_req[1];
    }
    const int64_t TH = (rows - k + 1) / 4 * 4;
    const int64_t RH = TH + k - 1;
    p.TH = (int)TH;
    p.tiles_y = (int)cdiv(H, TH);
    p.tiles_x = (int)cdiv(W, 64);
    // a row-pass unit reads ceil((d + 8 + k - 1) / 4) 16-byte groups from column 8 cg on
    const int64_t nwr = cdiv((p.c4 - c) + 8 + k - 1, 4);
    p.PI = (int)(round_up(56 + 4 * nwr, 8) + 4);          // pitches of 4 mod 8 floats: see the kernel
    p.PM = p.PI;                                          // the row-pass result replaces the staged input
    p.lds_bytes = (int)((RH * p.PI + 8 * cdiv(k, 4)) * 4);
    if (p.lds_bytes > LDS_LIMIT) return MERIT_ERR_UNSUPPORTED;
    const int64_t grid = N * p.tiles_y * p.tiles_x;
    if (grid >= INT_LIMIT || !fastdiv_ok(grid, p.tiles_x) || !fastdiv_ok(N * p.tiles_y, p.tiles_y) ||
        !fastdiv_ok(8 * RH, RH))
        return MERIT_ERR_UNSUPPORTED;
    p.div_tiles_x = make_fastdiv((uint32_t)p.tiles_x);
    p.div_tiles_y = make_fastdiv((uint32_t)p.tiles_y);
    p.div_rh = make_fastdiv((uint32_t)RH);

    pl->out_ndim = 3;
    pl->out_shape[0] = N; pl->out_shape[1] = H; pl->out_shape[2] = W;
    merit_launch_info &li = pl->info;
    li.kernel = "merit_sepfilter_tile";
    // persistent grid: the launcher sizes it from the device's CU count (256 on MI355X)
    p.wg_per_cu = (int)(LDS_LIMIT / p.lds_bytes);
    if (p.wg_per_cu > 8) p.wg_per_cu = 8;
    li.grid[0] = grid < 256 * p.wg_per_cu ? grid : 256 * p.wg_per_cu; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = p.lds_bytes;
    li.tile[0] = 1; li.tile[1] = TH; li.tile[2] = 64; li.tile[3] = k; li.tile[4] = k;
    return MERIT_OK;
}

// --------------------------------------------------------- bilateral filter ---
merit_status derive_bilateral(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_F32 || d.pad != MERIT_PAD_CLAMP) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 3 || d.n_acc != 2) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 3 || d.b.ndim != 1) return MERIT_ERR_UNSUPPORTED;
    const int64_t N = d.a.shape[0], H = d.a.shape[1], W = d.a.shape[2], k = d.b.shape[0];
    if (N < 0 || H <= 0 || W <= 0 || k <= 0) return MERIT_ERR_INVALID_ARG;
    const int64_t c = k / 2;
    const int axis_x[5] = {0, 1, 2, 1, 2};
    const int64_t stride_x[5] = {1, 1, 1, 1, 1};
    const int64_t offset_x[5] = {0, 0, 0, -c, -c};
    const int axis_k[5] = {MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 0};
    const int64_t stride_k[5] = {0, 0, 0, 0, 1};
    const int64_t offset_k[5] = {0, 0, 0, 0, 0};
    if (!operand_is(d.a, 5, axis_x, stride_x, offset_x)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 5, axis_k, stride_k, offset_k)) return MERIT_ERR_UNSUPPORTED;
    if (d.range[0] != N || d.range[1] != H || d.range[2] != W || d.range[3] != k || d.range[4] != k)
        return MERIT_ERR_SHAPE;
    if (k > 32 || H * W >= INT_LIMIT || N * H * W >= (1ll << 40)) return MERIT_ERR_UNSUPPORTED;

    BilatParams &p = pl->bil;
    p.N = (int)N; p.H = (int)H; p.W = (int)W; p.k = (int)k; p.c = (int)c;
    p.c4 = (int)round_up(c, 4);
    p.tiles_y = (int)cdiv(H, 16);
    p.tiles_x = (int)cdiv(W, 64);
    p.PI = (int)round_up(64 + p.c4 + (k - 1 - c), 4);
    const int64_t RH = 16 + k - 1;
    p.lds_bytes = (int)((RH * p.PI + 2 * k + 4) * 4);     // + one 16-byte group: whole-group reads of the last row
    p.scale = 0.0f; p.neg = 1;
    const int64_t grid = N * p.tiles_y * p.tiles_x;
    if (grid >= INT_LIMIT || !fastdiv_ok(grid, p.tiles_x) || !fastdiv_ok(N * p.tiles_y, p.tiles_y) ||
        !fastdiv_ok(RH * p.PI, p.PI / 4))
        return MERIT_ERR_UNSUPPORTED;
    p.div_tiles_x = make_fastdiv((uint32_t)p.tiles_x);
    p.div_tiles_y = make_fastdiv((uint32_t)p.tiles_y);
    p.div_p4 = make_fastdiv((uint32_t)(p.PI / 4));

    pl->out_ndim = 3;
    pl->out_shape[0] = N; pl->out_shape[1] = H; pl->out_shape[2] = W;
    merit_launch_info &li = pl->info;
    li.kernel = k <= 16 ? "merit_bilateral_rows" : "merit_bilateral_tile";   // four outputs along a row / down a column
    li.grid[0] = grid; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = p.lds_bytes;
    li.tile[0] = 1; li.tile[1] = 16; li.tile[2] = 64; li.tile[3] = k; li.tile[4] = k;
    return MERIT_OK;
}

// -------------------------------------------------------------- convolution ---
merit_status derive_conv(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_F16 || d.pad != MERIT_PAD_ZERO) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 4 || d.n_acc != 3) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 4 || d.b.ndim != 4) return MERIT_ERR_UNSUPPORTED;
    const int64_t DC = INT64_MIN;
    const int axis_x[7] = {0, MERIT_AXIS_UNUSED, 2, 3, 1, 2, 3};
    const int64_t stride_x[7] = {1, 0, DC, DC, 1, DC, DC};      // window strides = dilation
    const int64_t offset_x[7] = {0, 0, 0, 0, 0, DC, DC};
    const int axis_w[7] = {MERIT_AXIS_UNUSED, 0, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1, 2, 3};
    const int64_t stride_w[7] = {0, 1, 0, 0, 1, 1, 1};
    const int64_t offset_w[7] = {0, 0, 0, 0, 0, 0, 0};
    if (!operand_is(d.a, 7, axis_x, stride_x, offset_x)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 7, axis_w, stride_w, offset_w)) return MERIT_ERR_UNSUPPORTED;

    const int64_t N = d.a.shape[0], Cin = d.a.shape[1], H = d.a.shape[2], W = d.a.shape[3];
    const int64_t Cout = d.b.shape[0], kh = d.b.shape[2], kw = d.b.shape[3];
    const int64_t sh = d.a.stride[2], sw = d.a.stride[3];
    const int64_t dh = d.a.stride[5], dw = d.a.stride[6];
    const int64_t ph = -d.a.offset[5], pw = -d.a.offset[6];
    const int64_t OH = d.range[2], OW = d.range[3];
    if (N < 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0 || dh <= 0 || dw <= 0)
        return MERIT_ERR_INVALID_ARG;
    const int64_t eh = (kh - 1) * dh + 1, ew = (kw - 1) * dw + 1;      // extent of the dilated window
    if (d.b.shape[1] != Cin || d.range[0] != N || d.range[1] != Cout || d.range[4] != Cin ||
        d.range[5] != kh || d.range[6] != kw)
        return MERIT_ERR_SHAPE;
    if (H + 2 * ph < eh || W + 2 * pw < ew) return MERIT_ERR_SHAPE;
    if (OH != out_extent(H, eh, sh, ph) || OW != out_extent(W, ew, sw, pw)) return MERIT_ERR_SHAPE;
    if (N * Cin * H * W >= (1ll << 40) || OH * OW >= (1 << 24) || Cin > 4096 || Cout > 65535 * 32 ||
        kh > 31 || kw > 31 || sh > 16 || sw > 16 || dh > 16 || dw > 16)
        return MERIT_ERR_UNSUPPORTED;
    const bool dilated = dh != 1 || dw != 1;

    ConvParams &p = pl->conv;
    p.N = (int)N; p.Cin = (int)Cin; p.H = (int)H; p.W = (int)W; p.Cout = (int)Cout;
    p.relu = (d.op == MERIT_OP_CONV_DOT_RELU || d.op == MERIT_OP_CONV_DOT_RELU_POOLMAX ||
              d.op == MERIT_OP_CONV_DOT_ADD_RELU) ? 1 : 0;
    p.residual = (d.op == MERIT_OP_CONV_DOT_ADD || d.op == MERIT_OP_CONV_DOT_ADD_RELU) ? 1 : 0;
    const bool pool = d.op == MERIT_OP_CONV_DOT_POOLMAX || d.op == MERIT_OP_CONV_DOT_RELU_POOLMAX;
    p.pool = pool ? 1 : 0;
    p.PH = p.PW = p.PB = p.NB = p.pw8 = 0; p.pool_halo = 0;
    // fused pooling: a workgroup's tile is an even number of whole output rows (at least two)
    if (pool && (OH % 2 != 0 || OW % 2 != 0 || 2 * OW > 256)) return MERIT_ERR_UNSUPPORTED;
    p.OH = (int)OH; p.OW = (int)OW; p.kh = (int)kh; p.kw = (int)kw; p.sh = (int)sh; p.sw = (int)sw;
    p.ph = (int)ph; p.pw = (int)pw; p.dh = (int)dh; p.dw = (int)dw;

    const int64_t ohw = OH * OW;
    const int64_t ncb = cdiv(Cout, 32);
    p.CB = ncb >= 2 ? 2 : 1;
    // A grid that would leave more than half of the 256 CUs idle gets 32-channel blocks, i.e. twice
    // the workgroups (channel-block kernels; 8x128x56x56 -> 128, 3x3 / s2: 112 -> 224 workgroups,
    // 24.4 -> 14.5 us; with more workgroups than that the 64-channel blocks win: half the input staging).
    if (ncb >= 2 && Cin >= 8 && !pool && N * cdiv(ohw, 128) * cdiv(ncb, 2) <= 128) p.CB = 1;
    p.co_groups = (int)cdiv(ncb, p.CB);

    // try both tile sizes for a variant; prefer 256 pixels when the grid stays large
    // an explicit tile request selects the plain kernels; so does the residual layer (the added
    // tensor is staged by the wavefronts that also multiply)
    bool want_ws = pl->tile_req[2] <= 0 && !p.residual;
    auto try_variant = [&](int variant, int pxw, int nw) -> bool {
        ConvParams q = p;
        q.variant = variant;
        q.nchunks = 1; q.pipe = 0;
        q.PXW = pxw;
        q.NW = nw;
        q.TM = nw * pxw * 32;
        q.tiles_per_image = (int)cdiv(ohw, q.TM);
        q.rows_out_max = (int)((q.TM + OW - 2) / OW + 1);
        if (q.rows_out_max > OH) q.rows_out_max = (int)OH;
        q.tile_px = q.TM;
        if (pool) q.rows_out_max = 2;
        q.RHa = (int)((q.rows_out_max - 1) * sh + eh);
        if (variant == CONV_PLANAR_SMALLC) {
            if (kw > 16 || pw > 8 || dilated) return false;      // its fragments are runs of adjacent taps
            if (Cin * H * W * 2 >= (1ll << 31) || Cout * Cin * kh * kw * 2 >= (1ll << 31)) return false;    // byte offsets into an image / the weights
            q.padl = 8;
            // with an even column stride every window starts on the same column parity; if that
            // parity is odd and a slot is free, start the fragment one column earlier (front = 1)
            // so that it is dword-aligned in LDS and needs no funnel shift
            const bool odd_start = ((q.padl - pw) & 1) != 0;
            q.front = (sw % 2 == 0 && odd_start && kw != 8 && kw != 16) ? 1 : 0;
            q.aligned = (sw % 2 == 0 && ((q.padl - pw - q.front) & 1) == 0) ? 1 : 0;
            // a window row of more than 8 slots is two K-groups (two adjacent fragments)
            const int64_t parts = (q.front + kw > 8) ? 2 : 1;
            int64_t pitch = q.padl + W;
            const int64_t reach = q.padl - pw + (OW - 1) * sw + 2 + 8 * parts;
            if (reach > pitch) pitch = reach;
            q.pitch = (int)round_up(pitch, 8);
            q.G = (int)(Cin * kh * parts);
            q.G2 = (int)round_up(q.G, 2);
            q.S = q.G2 / 2;
            q.nchi = 0;
            q.lds_w_bytes = q.CB * q.G2 * 32 * 16;
            q.lds_x_bytes = (int)(Cin * q.RHa * q.pitch * 2);
            if (!fastdiv_ok((int64_t)Cin * q.RHa * (q.pitch / 8), q.pitch / 8)) return false;
            if (!fastdiv_ok((int64_t)Cin * q.RHa, q.RHa) || !fastdiv_ok(q.G2, kh)) return false;
            q.div_pitch8 = make_fastdiv((uint32_t)(q.pitch / 8));
            q.div_kh = make_fastdiv((uint32_t)kh);
            if (!fastdiv_ok((int64_t)q.CB * 32 * q.G2, q.G2)) return false;
            q.div_g2 = make_fastdiv((uint32_t)q.G2);
            q.lds_o_offset = (int)round_up((int64_t)q.lds_w_bytes + 32 + q.lds_x_bytes, 16);
        } else {
            q.front = 0; q.aligned = 0;
            q.padl = (int)pw;
            int64_t pitch = q.padl + W;
            const int64_t reach = (OW - 1) * sw + ew;
            if (reach > pitch) pitch = reach;
            q.pitch = (int)pitch;
            q.G = q.G2 = 0;
            // Channel groups of 8, an even number (the two halves of a wavefront take one each per
            // MFMA step).  All of them are staged at once when weights + input rows + output
            // staging fit in LDS; else the channels go through in passes of the largest even
            // group count that fits half of it (two workgroups per CU overlap staging and MFMAs),
            // or all of it if not even one pair fits the half.
            const int64_t nchi_all = cdiv(Cin, 16) * 2;
            const int64_t per_pair = kh * kw * q.CB * 64 * 16 + 2 * (int64_t)q.RHa * pitch * 16;
            const int64_t o_bytes = (int64_t)q.CB * 32 * (q.TM / 2 + 2) * 4;
            int64_t pairs = nchi_all / 2;
            q.pipe = 0;
            if (pairs * per_pair + o_bytes > LDS_LIMIT) {
                pairs = (LDS_LIMIT / 2 - o_bytes) / per_pair;
                if (pairs < 1) pairs = (LDS_LIMIT - o_bytes) / per_pair;
                if (pairs < 1) return false;
                // 3x3 and 1x1 layers with Cin % 8 == 0 get the pipelined form of the multi-pass
                // kernel (a pass's loads fly under the previous pass's MFMAs): a pass then is
                // at most 1 (3x3) or 2 (1x1) weight units (8 channels x all taps of an output
                // channel) and 1 input unit of 8 channels x 8 pixels (3 of 8 x 1 when W % 8 != 0) per thread.
                const int64_t T = kh * kw;
                if ((T == 9 || T == 1) && (Cin % 8) == 0) {
                    int64_t pp = pairs;
                    const int64_t by_w = (T == 9 ? 256 : 512) / (q.CB * 32 * 2);
                    // input: one 8-pixel unit per thread (W % 8 == 0), else three 1-pixel units
                    const int64_t by_x = (W % 8) == 0 ? 256 / (2 * q.RHa * (W / 8)) : 768 / (2 * q.RHa * W);
                    if (pp > by_w) pp = by_w;
                    if (pp > by_x) pp = by_x;
                    if (pp >= 1 && fastdiv_ok(768, W)) { pairs = pp; q.pipe = (int)T; q.div_w = make_fastdiv((uint32_t)W); }
                }
                // equal passes (the last one is padded with zero channels otherwise)
                const int64_t passes = cdiv(nchi_all / 2, pairs);
                pairs = cdiv(nchi_all / 2, passes);
            }
            q.nchi = (int)(2 * pairs);
            q.nchunks = (int)cdiv(nchi_all, q.nchi);
            q.S = (int)((q.nchi / 2) * kh * kw);
            q.lds_w_bytes = q.S * q.CB * 64 * 16;
            q.lds_x_bytes = (int)((int64_t)q.nchi * q.RHa * q.pitch * 16);
            if ((W % 8) == 0) {
                if (!fastdiv_ok((int64_t)q.nchi * q.RHa * (W / 8), W / 8)) return false;
                q.div_w8 = make_fastdiv((uint32_t)(W / 8));
            }
            if (!fastdiv_ok((int64_t)q.nchi * q.RHa, q.RHa)) return false;
            if (!fastdiv_ok((int64_t)q.CB * 32 * q.nchi, q.nchi)) return false;
            q.div_nchi = make_fastdiv((uint32_t)q.nchi);
            q.lds_o_offset = q.lds_w_bytes + q.lds_x_bytes;
        }
        q.lds_o_bytes = q.CB * 32 * (q.TM / 2 + 2) * 4;   // [channel][TM/2 + 2] dwords
        {
            const int64_t end_x = (int64_t)q.lds_w_bytes + (variant == CONV_PLANAR_SMALLC ? 32 : 0) + q.lds_x_bytes;
            const int64_t end_o = (int64_t)q.lds_o_offset + q.lds_o_bytes;
            q.lds_total = (int)round_up(end_x > end_o ? end_x : end_o, 16);
        }
        q.div_rha = make_fastdiv((uint32_t)q.RHa);
        // wave-specialised planar kernel: 4 multiplier + 4 mover wavefronts, double-buffered
        // input tile and output staging, one workgroup per CU
        q.ws = 0; q.su = 0; q.lg_chunks = 0;
        // (the kernel fetches a channel's weights in 16-byte vectors: at least one per channel)
        int lgc = 0;
        while ((1 << lgc) < q.pitch / 8) ++lgc;
        // (rows or output planes that start on any element: funnel-shifted staging and stores on the
        // output's 16-byte grid, not with the fused pooling)
        const int unal = ((W % 8) != 0 || (OH * OW) % 8 != 0) ? 1 : 0;
        q.unal = 0;
        if (variant == CONV_PLANAR_SMALLC && want_ws && q.front + kw <= 8 && pxw == 2 && nw == 4 && (!unal || !pool) && lgc <= 7 &&
            (((int64_t)Cin * q.RHa) << lgc) <= 128 * 10 && (int64_t)q.G * kw >= 8 &&
            N * Cin * H * W * 2 < (1ll << 31) &&
            N * Cout * OH * OW * 2 / (pool ? 4 : 1) < (1ll << 31)) {
            static const int steps[] = {4, 6, 8, 11, 12};
            int su = 0;
            for (int k = 0; k < 5 && !su; ++k)
                if (q.S <= steps[k] && q.S + 2 >= steps[k]) su = steps[k];
            const int64_t o_off = (int64_t)q.lds_w_bytes + 32 + 2 * (int64_t)q.lds_x_bytes;
            if (su && o_off + 2 * (int64_t)q.lds_o_bytes <= LDS_LIMIT) {
                q.ws = 1;
                q.unal = unal;
                // output planes off the 16-byte grid: tiles advance by 248 pixels and compute 256, so that
                // every 16-byte unit of a plane lies inside the tile that owns its first pixel
                // (unless the extra tiles cost the persistent grid, one workgroup per compute unit, a round that
                // outweighs the 12 % or so that such a tile's stores gain)
                if (unal && (OH * OW) % 8 != 0) {
                    const int64_t t_ov = std::max<int64_t>(1, cdiv(ohw - 8, q.TM - 8));
                    const int64_t slots = std::max<int64_t>(1, 256 / q.co_groups);
                    if (0.88 * (double)cdiv(N * t_ov, slots) <= (double)cdiv(N * q.tiles_per_image, slots)) {
                        q.tile_px = q.TM - 8;
                        q.tiles_per_image = (int)t_ov;
                    }
                }
                q.su = su;
                q.lg_chunks = lgc;
                q.lds_o_offset = (int)o_off;
                q.lds_total = (int)(o_off + 2 * (int64_t)q.lds_o_bytes);
            }
        }
        // the few-channel kernel without wave specialisation on output planes off the 16-byte grid: the same
        // overlapping tiles (a tile's run of a channel then has no elements outside every 16-byte store unit)
        if (variant == CONV_PLANAR_SMALLC && !q.ws && !pool && (OH * OW) % 8 != 0) {
            const int64_t t_ov = std::max<int64_t>(1, cdiv(ohw - 8, q.TM - 8));
            const int64_t wgs = std::min<int64_t>(3, LDS_LIMIT / (int64_t)conv_lds_bytes(q));
            const int64_t slots = std::max<int64_t>(1, 256 * wgs / q.co_groups);
            if (0.88 * (double)cdiv(N * t_ov, slots) <= (double)cdiv(N * q.tiles_per_image, slots)) {
                q.tile_px = q.TM - 8;
                q.tiles_per_image = (int)t_ov;
            }
        }
        if ((int64_t)conv_lds_bytes(q) > LDS_LIMIT) return false;
        q.wg_per_cu = (int)(LDS_LIMIT / (int64_t)conv_lds_bytes(q));
        // register budget: three workgroups (waves per SIMD) for the planar kernel, two otherwise
        const int reg_cap = q.ws ? 1 : (variant == CONV_PLANAR_SMALLC ? 3 : 2);
        if (q.wg_per_cu > reg_cap) q.wg_per_cu = reg_cap;
        if (!fastdiv_ok(ohw, OW) || !fastdiv_ok((int64_t)N * q.tiles_per_image, q.tiles_per_image)) return false;
        q.div_ow = make_fastdiv((uint32_t)OW);
        q.div_tiles = make_fastdiv((uint32_t)q.tiles_per_image);
        p = q;
        return true;
    };

    // Wave-specialised multi-pass kernel (conv2d_chws.hip): 256-pixel tiles x `cb` 32-channel blocks
    // (4 or 2), 16 input channels per pass through two LDS buffers, 3x3, 1x1 or 5x5 windows on a multiple
    // of 8 input channels.
    auto try_chws = [&](int cb, bool forced, int nw = 8, int tm = 256, bool halo = false) -> bool {
        const bool k5 = kh == 5 && kw == 5;
        if (!((kh == 3 && kw == 3) || (kh == 1 && kw == 1) || k5)) return false;
        // 5x5 windows: the 256 x 64 tiling on 8 wavefronts, no added tensor, no pooling
        if (k5 && (cb != 2 || nw != 8 || tm != 256 || pool || p.residual)) return false;
        // its tiles are 256 pixels of one image: small images (13x13, 7x7) would leave a third
        // and more of every tile empty and stay with the 128-pixel tiles of the plain kernels
        if (!forced && !pool && 4 * ohw < 3 * cdiv(ohw, tm) * tm) return false;
        if (Cin % 8 != 0 || Cin < 16 || (pool && p.residual) || ncb < 2) return false;
        // residual layer: 3x3 and 1x1 windows, the 64-channel tilings on 8 wavefronts
        if (p.residual && (!(kh == 3 || kh == 1) || cb != 2 || nw != 8)) return false;
        if (cb != 1 && cb != 2 && cb != 4) return false;
        // 32-channel tiles: 128 pixels on 8 wavefronts, 3x3 and 1x1 windows, no added tensor, no pooling (for launches
        // that would otherwise leave half the chip idle)
        if (cb == 1 && (nw != 8 || tm != 128 || pool || p.residual || k5)) return false;
        // fused pooling: 3x3 windows, the 64-channel tilings and the 128-channel one on 12 wavefronts; a tile is whole rows
        if (pool && (kh != 3 || !((cb == 2 && nw == 8) || (cb == 4 && nw == 12)) || (halo ? 3 : 2) * OW > tm)) return false;
        ConvParams q = p;
        q.variant = CONV_CHWS;
        q.CB = cb;
        q.co_groups = (int)cdiv(ncb, cb);
        q.PXW = tm == 128 ? 1 : ((cb == 4 && nw == 8) ? 4 : 2);    // 32-pixel blocks per multiplying wavefront
        q.NW = nw;                               // 8: four multiplying + four moving wavefronts; 12: eight + four
        q.TM = tm;                               // 256 pixels, or 128 (64- and 32-channel tiles on 8 wavefronts only)
        if (tm != 256 && !(tm == 128 && (cb == 2 || cb == 1) && nw == 8)) return false;
        q.tiles_per_image = (int)cdiv(ohw, q.TM);
        q.rows_out_max = (int)((q.TM + OW - 2) / OW + 1);
        if (q.rows_out_max > OH) q.rows_out_max = (int)OH;
        q.tile_px = q.TM;
        q.xq = 0;
        if (!pool && tm == 256) {
            // A tile of TM consecutive pixels starts anywhere in a row, so its covering sub-tensor
            // (Section IV-A, Eq. 9) is rows_out_max whole rows + the window's: on a 224-wide image
            // 5 staged rows for 1.14 rows of results.  Tiles of whole rows (R rows, R OW <= TM, the
            // rest of the MFMA tile idle) stage R - 1 + kh rows: taken when at least 80 % of the
            // tile is used and a fifth less input is staged over the image (224-wide: 51.8 -> 45.5 us for
            // 64 -> 64 channels; 112-wide: 3-5 % faster; 56-wide, a fifth less: no gain, not taken;
            // nor on the 128-pixel tiles of small launches, where the extra workgroups cost more).
            int64_t R = q.TM / OW;
            if (R > OH) R = OH;
            if (R >= 1 && (R * OW) % 8 == 0 && R * OW * 10 >= (int64_t)q.TM * 8) {
                const int64_t stage_lin = (int64_t)q.tiles_per_image * ((q.rows_out_max - 1) * sh + eh);
                const int64_t stage_row = cdiv(OH, R) * ((R - 1) * sh + eh);
                if (stage_row * 100 <= stage_lin * 80) {
                    q.tile_px = (int)(R * OW);
                    q.tiles_per_image = (int)cdiv(OH, R);
                    q.rows_out_max = (int)R;
                }
            }
        }
        if (pool) {
            // R whole rows per tile.  Carried row above (R even, R / 2 pooled rows per tile): bands of PB
            // pooled rows, a multiple of R / 2, about one band per compute unit (every band below the
            // first computes a tile more).  Computed row above (R odd, (R - 1) / 2 pooled rows): a
            // band is one tile.
            int64_t R = q.TM / OW;
            if (halo) { if (R % 2 == 0) --R; if (R > OH + 1) R = OH + 1; }
            else { R &= ~1ll; if (R > OH) R = OH; }
            const int64_t hp = R / 2;
            q.rows_out_max = (int)R;
            q.pool_halo = halo ? 1 : 0;
            q.PH = (int)(OH / 2); q.PW = (int)(OW / 2);
            int64_t nb = 256 / (N * q.co_groups);
            if (nb < 1) nb = 1;
            int64_t pb = halo ? hp : round_up(cdiv(q.PH, nb), hp);
            q.PB = (int)pb;
            q.NB = (int)cdiv(q.PH, pb);
            q.pw8 = (int)cdiv(q.PW, 4);                       // units of 4 pooled pixels per pooled row
            if (!fastdiv_ok(N * q.NB, q.NB) || !fastdiv_ok((hp + 1) * q.pw8, q.pw8)) return false;
            q.div_nb = make_fastdiv((uint32_t)q.NB);
            q.div_pw8 = make_fastdiv((uint32_t)q.pw8);
        }
        q.RHa = (int)((q.rows_out_max - 1) * sh + eh);
        // a window one row high with a row stride uses every sh-th image row: only those are staged
        q.row_skip = (kh == 1 && sh > 1 && !pool) ? 1 : 0;
        if (q.row_skip) q.RHa = q.rows_out_max;
        q.front = 0; q.aligned = 0; q.ws = 0; q.su = 0; q.lg_chunks = 0; q.pipe = 0; q.unal = 0;
        q.G = q.G2 = 0;
        q.padl = (int)pw;
        int64_t pitch = q.padl + W;
        const int64_t reach = (OW - 1) * sw + ew;
        if (reach > pitch) pitch = reach;
        pitch |= 1;                               // odd: staged rows start in different LDS bank groups
        q.pitch = (int)pitch;
        // 16 input channels per pass; 32 with the small tile, whose passes would otherwise be
        // shorter than the memory round trip that brings the next one
        int64_t ng = tm == 128 ? 2 : 1;
        if (kh == 1 && kw == 1 && Cin >= 128 && !pool) {
            // 1x1 windows: a pass is one tap; 64 channels per pass where its rows and staging units fit
            const int64_t g = 4, xb = 2 * g * (int64_t)q.RHa * pitch * 16, wb = g * cb * 64 * 16;
            const int64_t rows = 2 * g * (int64_t)q.RHa;
            const int64_t nu = (W % 8) == 0 ? rows * (W / 8) : ((W % 4) == 0 ? rows * (W / 4) : rows * W);
            const int64_t cap = ((W % 8) == 0 ? 2 : ((W % 4) == 0 ? (nw == 8 ? 4 : 2) : (nw == 8 ? 8 : 4))) * 256;
            if (2 * (wb + xb) <= LDS_LIMIT && nu <= cap) ng = g;
        }
        q.nchi = (int)(2 * ng);
        q.nchunks = (int)cdiv(Cin, 16 * ng);
        q.S = (int)(ng * kh * kw);
        const int64_t w_bytes = ng * kh * kw * cb * 64 * 16;
        const int64_t x_bytes = 2 * ng * (int64_t)q.RHa * pitch * 16;
        const int64_t o_bytes = (int64_t)cb * 32 * (q.TM / 2 + 2) * 4;
        const int64_t total = 2 * (w_bytes + x_bytes) > o_bytes ? 2 * (w_bytes + x_bytes) : o_bytes;
        if (total > LDS_LIMIT) return false;
        q.lds_w_bytes = (int)w_bytes; q.lds_x_bytes = (int)x_bytes; q.lds_buf_bytes = (int)(w_bytes + x_bytes);
        q.lds_o_offset = 0; q.lds_o_bytes = (int)o_bytes; q.lds_total = (int)total;
        if (pool) {
            // two carry buffers (the last row of a tile, every channel) behind the pass buffers / staging area
            const int64_t carry = 2 * (int64_t)cb * 32 * (OW / 2) * 4 + 16;
            q.lds_o_offset = (int)round_up(total, 16);
            q.lds_total = (int)(q.lds_o_offset + carry);
            if (q.lds_total > LDS_LIMIT) return false;
        }
        // staging units per moving thread and pass: 8 channels x 8 pixels (two at most), or x 1 pixel (eight; four on 12 wavefronts and for 5x5 windows)
        if ((W % 8) == 0) {
            const int64_t nu = 2 * ng * (int64_t)q.RHa * (W / 8);
            if (nu > 2 * 256 || !fastdiv_ok(nu, 2 * ng * (int64_t)q.RHa)) return false;
            q.xu = (int)cdiv(nu, 256);
            q.div_w8 = make_fastdiv((uint32_t)(W / 8));
            q.div_r2 = make_fastdiv((uint32_t)(2 * ng * q.RHa));
        } else if ((W % 4) == 0 && !k5) {
            // 8 channels x 4 pixels: four units per moving thread, two on 12 wavefronts
            const int64_t nu = 2 * ng * (int64_t)q.RHa * (W / 4);
            if (nu > (nw == 8 ? 4 : 2) * 256 || !fastdiv_ok(nu, 2 * ng * (int64_t)q.RHa)) return false;
            q.xu = (int)cdiv(nu, 256);
            q.xq = 1;
            q.div_r2 = make_fastdiv((uint32_t)(2 * ng * q.RHa));
        } else if ((W % 2) == 0 && !k5 && !pool && !p.residual && 2 * ng * (int64_t)q.RHa * (W / 2) <= (nw == 8 ? 8 : 4) * 256 &&
                   fastdiv_ok(2 * ng * (int64_t)q.RHa * (W / 2), 2 * ng * (int64_t)q.RHa)) {
            // 8 channels x 2 pixels (rows of an even width start on 4-byte boundaries: 14x14 layers), eight units
            // per moving thread, four on 12 wavefronts
            q.xu = (int)cdiv(2 * ng * (int64_t)q.RHa * (W / 2), 256);
            q.xq = 2;
            q.div_r2 = make_fastdiv((uint32_t)(2 * ng * q.RHa));
        } else {
            const int64_t nu = 2 * ng * (int64_t)q.RHa * W;
            if (nu > ((nw == 8 && !k5) ? 8 : 4) * 256 || !fastdiv_ok(nu, W)) return false;
            q.xu = (int)cdiv(nu, 256);
            q.div_w = make_fastdiv((uint32_t)W);
        }
        const int64_t nitems = pool ? N * q.NB * q.co_groups : N * q.tiles_per_image * q.co_groups;
        if (nitems >= (1ll << 30) || !fastdiv_ok(nitems + 256, q.co_groups) || !fastdiv_ok(2 * ng * (int64_t)q.RHa, q.RHa) ||
            !fastdiv_ok(ohw, OW) || !fastdiv_ok(N * q.tiles_per_image, q.tiles_per_image))
            return false;
        if (N * Cin * H * W >= (1ll << 31) || N * Cout * ohw >= (1ll << 31)) return false;
        q.div_cog = make_fastdiv((uint32_t)q.co_groups);
        q.div_rha = make_fastdiv((uint32_t)q.RHa);
        q.div_ow = make_fastdiv((uint32_t)OW);
        q.div_tiles = make_fastdiv((uint32_t)q.tiles_per_image);
        q.wg_per_cu = 1;
        p = q;
        return true;
    };

    // tile = (wavefronts per workgroup) x (pixels per wavefront): 4 x 32, 4 x 64 or, for the
    // planar kernel, 8 x 32.  256-pixel tiles when that still leaves a large grid.
    const bool want_big = N * cdiv(ohw, 256) * p.co_groups >= 512;
    bool ok = false;
    pl->est_units = 0.0;
    pl->two_pass = 0;
    if (pool && Cin >= 8) {
        // many input channels: the wave-specialised multi-pass kernel pools out of its staging area.
        // A tile request names one of its tilings: 8 x 64 (256 pixels x 64 channels), 8 x 32 (128 x 64),
        // 12 x 64 (256 x 128).
        const bool req = pl->tile_req[2] > 0 && pl->tile_req[3] > 0;
        const int64_t rw = pl->tile_req[2], rp = pl->tile_req[3];
        if (req && !((rw == 8 && (rp == 64 || rp == 32)) || (rw == 12 && rp == 64))) return MERIT_ERR_UNSUPPORTED;
        // Six candidates: 256 x 64, 128 x 64 or 256 x 128 tiles, the row above a tile's first pooled
        // row carried from the tile before or computed by the tile itself.  Estimated time = rounds of
        // the grid x tiles per workgroup x cost of a tile (256 x 64: 1, 128 x 64: 0.6, 256 x 128: 1.6; from timings).
        int best_tm = 0, best_cb = 0; bool best_halo = false; double best = 0.0;
        for (int cand = 0; cand < 6; ++cand) {
            const int shape = cand >> 1;                       // 0: 256 x 64, 1: 128 x 64, 2: 256 x 128
            const int tm = shape == 1 ? 128 : 256, cb = shape == 2 ? 4 : 2, nw = shape == 2 ? 12 : 8;
            const bool halo = (cand & 1) != 0;
            if (req && !(rw == nw && rp == (shape == 1 ? 32 : 64))) continue;
            if (cb == 4 && ncb < 4) continue;
            const ConvParams saved = p;
            const bool fits = try_chws(cb, true, nw, tm, halo);
            const ConvParams q = p;
            p = saved;
            if (!fits) continue;
            const int64_t items = N * q.NB * q.co_groups;
            const int64_t hp = q.rows_out_max / 2;
            const int64_t per_item = cdiv(q.PB, hp) + (halo || q.NB == 1 ? 0 : 1);
            const double cost = (double)cdiv(items, 256) * (double)per_item * (shape == 0 ? 1.0 : (shape == 1 ? 0.6 : 1.6));
            if (!best_tm || cost < best) { best_tm = tm; best_cb = cb; best_halo = halo; best = cost; }
        }
        ok = best_tm != 0 && try_chws(best_cb, true, best_cb == 4 ? 12 : 8, best_tm, best_halo);
        if (!ok) return MERIT_ERR_UNSUPPORTED;
        pl->est_units = best;
    } else if (pool) {
        // few input channels: the wave-specialised planar kernel pools; a tile request must name it (8 x 64) or nothing
        if (pl->tile_req[2] > 0 && pl->tile_req[3] > 0 && (pl->tile_req[2] != 8 || pl->tile_req[3] != 64))
            return MERIT_ERR_UNSUPPORTED;
        if (OW % 16 != 0) return MERIT_ERR_UNSUPPORTED;    // it pools 8 columns at a time
        want_ws = true;
        ok = try_variant(CONV_PLANAR_SMALLC, 2, 4) && p.ws;
        if (!ok) return MERIT_ERR_UNSUPPORTED;
        p.PH = (int)(OH / 2); p.PW = (int)(OW / 2); p.pw8 = p.PW / 8;
        // bands of pooled rows: about one workgroup per compute unit, but at least 4 rows per
        // band (every band recomputes one convolution row pair above its first pooled row)
        int64_t nb = 256 / (N * p.co_groups > 0 ? N * p.co_groups : 1);
        const int64_t nb_max = p.PH >= 4 ? p.PH / 4 : 1;
        if (nb > nb_max) nb = nb_max;
        if (nb < 1) nb = 1;
        p.PB = (int)cdiv(p.PH, nb);
        p.NB = (int)cdiv(p.PH, p.PB);
        if (!fastdiv_ok((int64_t)N * p.NB, p.NB) || !fastdiv_ok((int64_t)128 * 2 * p.CB, p.pw8))
            return MERIT_ERR_UNSUPPORTED;
        p.div_nb = make_fastdiv((uint32_t)p.NB);
        p.div_pw8 = make_fastdiv((uint32_t)p.pw8);
        if ((int64_t)N * p.NB >= (1ll << 31)) return MERIT_ERR_UNSUPPORTED;
    } else if (pl->tile_req[2] > 0 && pl->tile_req[3] > 0) {
        const int64_t nw = pl->tile_req[2], ppw = pl->tile_req[3];
        if ((nw != 4 && nw != 8 && nw != 12) || (ppw != 32 && ppw != 64 && ppw != 128)) return MERIT_ERR_UNSUPPORTED;
        if (ppw == 128 && nw != 8) return MERIT_ERR_UNSUPPORTED;
        if (nw == 12) {
            // 8 multiplying (64 pixels x 64 channels each) + 4 moving wavefronts: 256 pixels x 128 channels
            if (ppw != 64 || Cin < 8) return MERIT_ERR_UNSUPPORTED;
            ok = try_chws(4, true, 12);
            if (!ok) return MERIT_ERR_UNSUPPORTED;
        } else if (nw == 8 && Cin >= 8) {
            // 4 multiplying + 4 moving wavefronts on many channels: 256 pixels x 128 (4 x 32) or 64 channels
            ok = ppw == 32 ? try_chws(2, true, 8, 128) : try_chws(ppw == 128 ? 4 : 2, true);
            if (!ok) return MERIT_ERR_UNSUPPORTED;
        } else if (ppw == 128) {
            return MERIT_ERR_UNSUPPORTED;
        } else if (nw == 8 && ppw == 64) {
            // 4 multiplier wavefronts x 64 pixels + 4 mover wavefronts: the wave-specialised kernel
            if (p.residual) return MERIT_ERR_UNSUPPORTED;
            want_ws = true;
            if (Cin < 8) ok = try_variant(CONV_PLANAR_SMALLC, 2, 4) && p.ws;
            if (!ok) return MERIT_ERR_UNSUPPORTED;
        } else if (Cin < 8) ok = try_variant(CONV_PLANAR_SMALLC, (int)(ppw / 32), (int)nw);
        if (!ok && nw == 4) ok = try_variant(CONV_CHBLOCK, (int)(ppw / 32), 4);
    } else {
        // window rows of 9 to 16 taps with more 128-pixel tiles than compute units: 256-pixel tiles on 8
        // wavefronts (8 x 3 x 227 x 227 -> 96, 11x11 / s4: 30.8 -> 20.9 us; 4 wavefronts x 64 pixels: 23.8)
        if (Cin < 8 && kw > 8 && N * cdiv(ohw, 128) * p.co_groups > 256) ok = try_variant(CONV_PLANAR_SMALLC, 1, 8);
        if (!ok && Cin < 8)
            ok = want_big ? (try_variant(CONV_PLANAR_SMALLC, 2, 4) || try_variant(CONV_PLANAR_SMALLC, 1, 4))
                          : (try_variant(CONV_PLANAR_SMALLC, 1, 4) || try_variant(CONV_PLANAR_SMALLC, 2, 4));
        if (!ok)
            ok = want_big ? (try_variant(CONV_CHBLOCK, 2, 4) || try_variant(CONV_CHBLOCK, 1, 4))
                          : (try_variant(CONV_CHBLOCK, 1, 4) || try_variant(CONV_CHBLOCK, 2, 4));
        // 3x3 layers on at least 32 input channels (a multiple of 8) and at least 33 output channels:
        // the wave-specialised multi-pass kernel.  Its tilings: 256 pixels x 128 channels on 12
        // wavefronts, 256 x 64 and 128 x 64 (32 channels per pass) on 8.  The one with the lowest
        // estimate rounds of the grid x cost of a tile (1.6, 1, 0.6 from timings) is taken, the larger
        // tile on a tie: few large tiles while they still fill the chip, else more small ones --
        // also for images far smaller than a tile (13x13 on 256-pixel tiles: 32 us, against 98 us on
        // the plain multi-pass kernel; 7x7 on 128-pixel tiles: 28 against 88).  1x1 layers the same
        // (256 -> 64 on 56x56: 8.1 against 11.9 us, 1024 -> 256 on 14x14: 27 against 51); with a residual
        // tensor from 128 input channels on (128 -> 512 on 28x28: 11.7 against 36 us; 64 -> 256 on 56x56 is
        // a single short pass and stays on the single-pass kernel: 12.7 against 14.0).
        if (((kh == 3 && kw == 3) || (kh == 1 && kw == 1 && (!p.residual || Cin >= 128)) || (kh == 5 && kw == 5 && !p.residual)) && Cin >= 32 && (Cin % 8) == 0 && ncb >= 2) {
            int best = -1; double best_cost = 0.0;
            for (int shape = 0; shape < 4; ++shape) {          // 0: 256 x 128 on 12 wavefronts, 1: 256 x 64, 2: 128 x 64, 3: 128 x 32
                if (shape == 0 && ncb < 4) continue;
                const int64_t tm = shape >= 2 ? 128 : 256;
                const int cbs = shape == 0 ? 4 : (shape == 3 ? 1 : 2);
                const ConvParams saved = p;
                const bool fits = try_chws(cbs, true, shape == 0 ? 12 : 8, (int)tm);
                const int64_t items = N * (int64_t)p.tiles_per_image * p.co_groups;     // (of the trial, if it fits)
                const double cost = (double)cdiv(items, 256) * (shape == 0 ? 1.6 : (shape == 1 ? 1.0 : (shape == 2 ? 0.6 : 0.42)));
                p = saved;
                if (fits && (best < 0 || cost < best_cost)) { best = shape; best_cost = cost; }
            }
            if (best >= 0 && try_chws(best == 0 ? 4 : (best == 3 ? 1 : 2), true, best == 0 ? 12 : 8, best >= 2 ? 128 : 256)) {
                ok = true;
                pl->est_units = best_cost;
            }
        }
    }
    if (!ok) {
        // neither MFMA kernel holds this shape's operands in LDS: the one-element-per-thread
        // kernel takes any shape (not a tile request, which names an MFMA tiling, and not the
        // fused pooling, which only the wave-specialised kernel does)
        if (pool || (pl->tile_req[2] > 0 && pl->tile_req[3] > 0)) return MERIT_ERR_UNSUPPORTED;
        const int64_t per_image = Cout * ohw;
        if (per_image >= INT_LIMIT || H * W >= INT_LIMIT || Cout * Cin * kh * kw >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;
        p.variant = CONV_DIRECT;
        // a workgroup: 256 pixels x a block of output channels; the channel blocks count as
        // tiles of the image here (grid.y stays 1)
        p.PXW = 1; p.NW = 4; p.TM = 256; p.CB = 1; p.ws = 0; p.su = 0;
        p.co_groups = (int)cdiv(Cout, conv_direct_channels());
        p.tiles_per_image = (int)(p.co_groups * cdiv(ohw, 256));
        p.rows_out_max = 1; p.RHa = (int)eh; p.pitch = (int)W; p.padl = 0;
        p.G = p.G2 = p.S = p.nchi = 0; p.nchunks = 1; p.pipe = 0;
        p.lds_w_bytes = p.lds_x_bytes = p.lds_o_offset = p.lds_o_bytes = 0;
        p.lds_total = 32 * 1024;          // the kernel's own (static) weight buffer
        p.front = p.aligned = p.lg_chunks = 0;
        p.wg_per_cu = 8;
        p.div_ow = make_fastdiv((uint32_t)OW);
        p.div_tiles = make_fastdiv((uint32_t)p.tiles_per_image);
    }
    if ((int64_t)N * p.tiles_per_image >= (1ll << 31)) return MERIT_ERR_UNSUPPORTED;

    pl->out_ndim = 4;
    pl->out_shape[0] = N; pl->out_shape[1] = Cout; pl->out_shape[2] = OH; pl->out_shape[3] = OW;
    if (pool) { pl->out_shape[2] = p.PH; pl->out_shape[3] = p.PW; }
    merit_launch_info &li = pl->info;
    li.kernel = conv_kernel_name(p);
    // persistent grid; the launcher sizes it from the device's CU count (256 on MI355X)
    {
        int64_t slots = 256 * (int64_t)p.wg_per_cu / p.co_groups;
        if (slots < 1) slots = 1;
        const int64_t nt = (int64_t)N * p.tiles_per_image;
        li.grid[0] = nt < slots ? nt : slots;
        if (pool) li.grid[0] = (int64_t)N * p.NB;          // one workgroup per band, not persistent
        if (p.variant == CONV_DIRECT) li.grid[0] = nt;     // one workgroup per 256 pixels x 8 channels
        if (p.variant == CONV_CHWS) li.grid[0] = nt * p.co_groups < 256 ? nt * p.co_groups : 256;   // (tile, channel block) items
        if (p.variant == CONV_CHWS && pool) {                                                       // (band, channel block) items
            const int64_t nb = (int64_t)N * p.NB * p.co_groups;
            li.grid[0] = nb < 256 ? nb : 256;
        }
    }
    li.grid[1] = (p.variant == CONV_DIRECT || p.variant == CONV_CHWS) ? 1 : p.co_groups; li.grid[2] = 1;
    li.block[0] = p.ws ? 512 : p.NW * 64; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = (int64_t)conv_lds_bytes(p);
    li.tile[0] = 1; li.tile[1] = p.CB * 32; li.tile[2] = p.rows_out_max; li.tile[3] = OW;
    li.tile[4] = Cin; li.tile[5] = kh; li.tile[6] = kw;
    // convolution rows a band computes: its own and the row pair (few-channel kernel) or tile above
    if (pool) li.tile[2] = p.variant == CONV_CHWS ? ((p.pool_halo || p.NB == 1) ? p.rows_out_max * (int)cdiv(p.PB, p.rows_out_max / 2) : 2 * p.PB + p.rows_out_max) : 2 * (p.PB + 1);

    // Convolution + pooling on many channels: pooling inside the kernel costs MFMA time (a band of
    // pooled rows below the first recomputes the tile above it, tiles are whole rows, the 128-channel
    // tiling rarely fits), which a compute-bound layer cannot hide.  When the estimate for the
    // plain convolution plus one pass of the binary16 pooling kernel over its result is clearly
    // lower, the plan runs as those two launches (the result is the same: the maxima are exact).
    // Estimates in microseconds: a launch 4, a 256 x 64 tile 1.5 + 0.058 Cin kh kw / 9 (from
    // timings on 64 .. 512 channels), the pooling pass 3.5 (it cannot start before the convolution
    // has drained) + 1.25 x the convolution's result at 2.9 TB/s (measured: + 9 us for 12.8 MB,
    // + 3.4 us for 1.6 MB).  A tile request names a fused tiling and keeps the plan fused.
    if (pool && p.variant == CONV_CHWS && !(pl->tile_req[2] > 0 && pl->tile_req[3] > 0) && pl->est_units > 0.0) {
        merit_plan *plain = new (std::nothrow) merit_plan(*pl);
        if (plain) {
            plain->desc.op = p.relu ? MERIT_OP_CONV_DOT_RELU : MERIT_OP_CONV_DOT;
            if (derive_conv(plain) == MERIT_OK && plain->conv.variant == CONV_CHWS && plain->est_units > 0.0) {
                const double unit = 1.5 + 0.058 * (double)Cin * (double)(kh * kw) / 9.0;
                const double conv_bytes = (double)N * (double)Cout * (double)ohw * 2.0;
                const double t_fused = 4.0 + pl->est_units * unit;
                const double t_two = 4.0 + plain->est_units * unit + 3.5 + 1.25 * conv_bytes / 2.9e6;
                // (on a short launch the second launch and the temporary's allocation calls cost
                // more host time than the GPU saves: the convolution alone must be estimated at 12 us)
                if (t_two < 0.9 * t_fused && plain->est_units * unit >= 12.0) {
                    pl->two_pass = 1;
                    pl->conv2 = plain->conv;
                    const int64_t keep2 = li.tile[2];
                    li = plain->info;
                    li.tile[2] = keep2;
                    li.kernel = "merit_conv2d_chws+merit_maxpool_f16";
                }
            }
            delete plain;
        }
    }
    return MERIT_OK;
}

// ----------------------------------------------------- depthwise convolution ---
merit_status derive_dw(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_F16 || d.pad != MERIT_PAD_ZERO) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 4 || d.n_acc != 2) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 4 || d.b.ndim != 3) return MERIT_ERR_UNSUPPORTED;
    const int64_t DC = INT64_MIN;
    const int axis_x[6] = {0, 1, 2, 3, 2, 3};
    const int64_t stride_x[6] = {1, 1, DC, DC, 1, 1};
    const int64_t offset_x[6] = {0, 0, 0, 0, DC, DC};
    const int axis_w[6] = {MERIT_AXIS_UNUSED, 0, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1, 2};
    const int64_t stride_w[6] = {0, 1, 0, 0, 1, 1};
    const int64_t offset_w[6] = {0, 0, 0, 0, 0, 0};
    if (!operand_is(d.a, 6, axis_x, stride_x, offset_x)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 6, axis_w, stride_w, offset_w)) return MERIT_ERR_UNSUPPORTED;
    const int64_t N = d.a.shape[0], C = d.a.shape[1], H = d.a.shape[2], W = d.a.shape[3];
    const int64_t OH = d.range[2], OW = d.range[3], kh = d.range[4], kw = d.range[5];
    const int64_t sh = d.a.stride[2], sw = d.a.stride[3];
    const int64_t ph = -d.a.offset[4], pw = -d.a.offset[5];
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
        return MERIT_ERR_INVALID_ARG;
    if (d.range[0] != N || d.range[1] != C || d.b.shape[0] != C || d.b.shape[1] != kh || d.b.shape[2] != kw)
        return MERIT_ERR_SHAPE;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return MERIT_ERR_SHAPE;
    if (OH != out_extent(H, kh, sh, ph) || OW != out_extent(W, kw, sw, pw)) return MERIT_ERR_SHAPE;
    if (N * C >= INT_LIMIT || H * W >= INT_LIMIT || kh > 31 || kw > 31 || sh > 16 || sw > 16)
        return MERIT_ERR_UNSUPPORTED;

    DwParams &p = pl->dw;
    p.NC = (int)(N * C); p.C = (int)C; p.H = (int)H; p.W = (int)W; p.OH = (int)OH; p.OW = (int)OW;
    p.kh = (int)kh; p.kw = (int)kw; p.sh = (int)sh; p.sw = (int)sw; p.ph = (int)ph; p.pw = (int)pw;
    if (kh == 3 && kw == 3 && sh == 1 && sw == 1 && ph == 1 && pw == 1 && (W % 8) == 0 && W <= 4096 &&
        pl->tile_req[2] <= 0) {
        p.variant = DW_ROWS_K3S1P1;
        int64_t TH = 4096 / W;                       // about two 8-pixel units per thread
        if (TH < 1) TH = 1;
        if (TH > OH) TH = OH;
        p.TH = (int)TH;
        p.pitch = (int)(W / 8 + 2);
        p.lds_w_offset = 0;
        p.lds_bytes = (int)((TH + 2) * p.pitch * 16);
        p.div_ow = make_fastdiv((uint32_t)(W / 8));
    } else {
        p.variant = DW_TILE_GENERIC;
        p.pitch = (int)(W + 2 * pw);
        int64_t TH = pl->tile_req[2] > 0 ? pl->tile_req[2] : (4096 / OW > 0 ? 4096 / OW : 1);
        if (TH > OH) TH = OH;
        while (TH > 1 && ((TH - 1) * sh + kh) * p.pitch * 2 > 48 * 1024) TH = (TH + 1) / 2;
        const int64_t RH = (TH - 1) * sh + kh;
        if (RH * p.pitch * 2 > 96 * 1024) return MERIT_ERR_UNSUPPORTED;      // very wide rows: no column tiling here
        p.TH = (int)TH;
        p.lds_w_offset = (int)round_up(RH * p.pitch * 2, 16);
        p.lds_bytes = (int)(p.lds_w_offset + kh * kw * 4);
        if (!fastdiv_ok(RH * p.pitch, p.pitch) || !fastdiv_ok(TH * OW, OW)) return MERIT_ERR_UNSUPPORTED;
        p.div_ow = make_fastdiv((uint32_t)OW);
    }
    p.tiles_y = (int)cdiv(OH, p.TH);
    const int64_t grid = (int64_t)p.NC * p.tiles_y;
    if (grid >= INT_LIMIT || !fastdiv_ok(grid, p.tiles_y) || !fastdiv_ok(p.NC, C) ||
        !fastdiv_ok((int64_t)(p.TH + 2 + kh * 16) * p.pitch, p.pitch))
        return MERIT_ERR_UNSUPPORTED;
    p.div_tiles_y = make_fastdiv((uint32_t)p.tiles_y);
    p.div_c = make_fastdiv((uint32_t)C);
    p.div_pitch = make_fastdiv((uint32_t)p.pitch);

    pl->out_ndim = 4;
    pl->out_shape[0] = N; pl->out_shape[1] = C; pl->out_shape[2] = OH; pl->out_shape[3] = OW;
    merit_launch_info &li = pl->info;
    li.kernel = dwconv_kernel_name(p);
    li.grid[0] = grid; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = p.lds_bytes;
    li.tile[0] = 1; li.tile[1] = 1; li.tile[2] = p.TH; li.tile[3] = OW; li.tile[4] = kh; li.tile[5] = kw;
    return MERIT_OK;
}

// -------------------------------------------------------- correlation layer ---
merit_status derive_corr(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    if (d.dtype != MERIT_F16 || d.pad != MERIT_PAD_ZERO) return MERIT_ERR_UNSUPPORTED;
    if (d.n_par != 5 || d.n_acc != 1) return MERIT_ERR_UNSUPPORTED;
    if (d.a.ndim != 4 || d.b.ndim != 4) return MERIT_ERR_UNSUPPORTED;
    const int64_t n = d.range[3];
    if (n <= 0 || (n % 2) == 0 || d.range[4] != n) return MERIT_ERR_SHAPE;
    const int64_t R = (n - 1) / 2;
    const int64_t sd = d.b.stride[3];
    if (sd <= 0) return MERIT_ERR_INVALID_ARG;
    const int axis_1[6] = {0, 2, 3, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1};
    const int64_t stride_1[6] = {1, 1, 1, 0, 0, 1};
    const int64_t offset_1[6] = {0, 0, 0, 0, 0, 0};
    const int axis_2[6] = {0, 2, 3, 2, 3, 1};
    const int64_t stride_2[6] = {1, 1, 1, sd, sd, 1};
    const int64_t offset_2[6] = {0, 0, 0, -R * sd, -R * sd, 0};
    if (!operand_is(d.a, 6, axis_1, stride_1, offset_1)) return MERIT_ERR_UNSUPPORTED;
    if (!operand_is(d.b, 6, axis_2, stride_2, offset_2)) return MERIT_ERR_UNSUPPORTED;
    const int64_t N = d.a.shape[0], C = d.a.shape[1], H = d.a.shape[2], W = d.a.shape[3];
    if (N < 0 || C <= 0 || H <= 0 || W <= 0) return MERIT_ERR_INVALID_ARG;
    for (int i = 0; i < 4; ++i)
        if (d.b.shape[i] != d.a.shape[i]) return MERIT_ERR_SHAPE;
    if (d.range[0] != N || d.range[1] != H || d.range[2] != W || d.range[5] != C) return MERIT_ERR_SHAPE;
    // the kernel stages 8-pixel units and gives a wavefront at most 8 column displacements
    if ((W % 8) != 0 || R > 15 || sd > 8 || C > 65536) return MERIT_ERR_UNSUPPORTED;
    if (N * C * H * W >= INT_LIMIT || N * H * W * n * n >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;

    CorrParams &p = pl->corr;
    p.N = (int)N; p.C = (int)C; p.H = (int)H; p.W = (int)W; p.R = (int)R; p.sd = (int)sd; p.n = (int)n;
    p.nchi = (int)cdiv(C, 8);
    p.xchunks = (int)cdiv(W, 64);
    p.lead = (int)round_up(R * sd, 8);
    p.cols2 = (int)round_up(64 + p.lead + R * sd, 8);
    // staged rows ordered by residue class of the column modulo sd (the 16 pixels of an MFMA block are adjacent)
    p.pitch1 = (int)cdiv(64, sd); p.P1 = (int)(sd * p.pitch1);
    p.pitch2 = (int)cdiv(p.cols2, sd); p.P2 = (int)(sd * p.pitch2);
    p.nsb = (int)cdiv(p.pitch1, 16); p.nblk = (int)(sd * p.nsb);
    p.nb = (int)cdiv(16 + 2 * R, 16);
    // channel groups per pass: whole reduction steps of 4 groups, at most two staging units per
    // thread, and about 40 KB so that four workgroups share a CU's LDS (measured best)
    const int64_t per_g_full = 8 + p.cols2 / 8;
    const int64_t per_group = ((int64_t)p.P1 + p.P2) * 16;
    int64_t chg = (CORR_LDS_KB * 1024) / per_group;
    if (chg > 256 * CORR_XB / per_g_full) chg = 256 * CORR_XB / per_g_full;
    chg = chg / 4 * 4;
    if (chg < 4) chg = 4;
    const int64_t nchi4 = round_up(p.nchi, 4);
    p.chg = (int)(chg < nchi4 ? chg : nchi4);
    if (p.chg * per_g_full > 256 * CORR_XB || p.chg * per_group > LDS_LIMIT) return MERIT_ERR_UNSUPPORTED;
    p.div_sd = make_fastdiv((uint32_t)sd);
    p.div_perg = make_fastdiv((uint32_t)per_g_full);
    p.div_perg_last = make_fastdiv((uint32_t)((W % 64) / 8 + p.cols2 / 8));
    const int64_t grid = N * H * n * p.xchunks;
    if (grid >= INT_LIMIT || !fastdiv_ok(grid, p.xchunks) || !fastdiv_ok(grid, n) || !fastdiv_ok(grid, H))
        return MERIT_ERR_UNSUPPORTED;
    p.xq = (int)(grid / 8); p.xr = (int)(grid % 8);
    p.div_xchunks = make_fastdiv((uint32_t)p.xchunks);
    p.div_n = make_fastdiv((uint32_t)n);
    p.div_h = make_fastdiv((uint32_t)H);

    pl->out_ndim = 5;
    pl->out_shape[0] = N; pl->out_shape[1] = H; pl->out_shape[2] = W; pl->out_shape[3] = n; pl->out_shape[4] = n;
    merit_launch_info &li = pl->info;
    li.kernel = "merit_corr_mfma";
    li.grid[0] = grid; li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = (int64_t)corr_lds_bytes(p);
    li.tile[0] = 1; li.tile[1] = 1; li.tile[2] = W < 64 ? W : 64; li.tile[3] = 1; li.tile[4] = n; li.tile[5] = C;
    return MERIT_OK;
}

// ------------------------------------------------ any descriptor (Eq. 1, Eq. 5) ---
// What none of the patterns above recognises still is a ranged inner product: the definition
// kernel (generic.hip) runs it, one thread per row.  Operations: the dot products (CONV_DOT,
// CONV_DOT_RELU, DWCONV_DOT, CORR_DOT: binary16, zero or clamp padding, two operands) and the
// single-operand reductions (POOL_MAX: any padding rule; POOL_AVG: exclude, zero or clamp; fp32).
// The output is the dense tensor of the parallel ranges, so there are at most MERIT_MAX_DIMS of them.
merit_status derive_generic(merit_plan *pl)
{
    const merit_plan_desc &d = pl->desc;
    GenericParams &g = pl->gen;
    std::memset(&g, 0, sizeof(g));
    switch (d.op) {
    case MERIT_OP_CONV_DOT:
    case MERIT_OP_CONV_DOT_RELU:
    case MERIT_OP_DWCONV_DOT:
    case MERIT_OP_CORR_DOT:
        if (d.dtype != MERIT_F16 || (d.pad != MERIT_PAD_ZERO && d.pad != MERIT_PAD_CLAMP) || d.b.ndim < 1)
            return MERIT_ERR_UNSUPPORTED;
        g.mode = 0;
        g.relu = d.op == MERIT_OP_CONV_DOT_RELU ? 1 : 0;
        break;
    case MERIT_OP_POOL_MAX:
        if (d.dtype != MERIT_F32) return MERIT_ERR_UNSUPPORTED;
        g.mode = 1;
        break;
    case MERIT_OP_POOL_AVG:
        if (d.dtype != MERIT_F32 || d.pad == MERIT_PAD_NEG_INF) return MERIT_ERR_UNSUPPORTED;
        g.mode = 2;
        break;
    default: return MERIT_ERR_UNSUPPORTED;
    }
    if (d.n_par > MERIT_MAX_DIMS) return MERIT_ERR_UNSUPPORTED;
    g.pad = (int)d.pad;
    g.n_par = d.n_par; g.n_acc = d.n_acc;
    const int nidx = d.n_par + d.n_acc;
    int64_t rows = 1, acc = 1;
    for (int j = 0; j < nidx; ++j) {
        const int64_t r = d.range[j];
        if (r >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;
        if (j >= d.n_par && r < 1) return MERIT_ERR_INVALID_ARG;     // an empty reduction has no value
        g.range[j] = (int)r;
        if (j < d.n_par) { rows *= r; if (rows >= (1ll << 38)) return MERIT_ERR_UNSUPPORTED; }
        else { acc *= r; if (acc >= (1ll << 40)) return MERIT_ERR_UNSUPPORTED; }
    }
    g.rows = rows; g.acc = acc;
    auto operand = [&](const merit_operand &o, GenericOperand &q) -> merit_status {
        q.ndim = o.ndim;
        int64_t elems = 1;
        for (int i = o.ndim - 1; i >= 0; --i) {
            if (o.shape[i] < 1 || o.shape[i] >= (1ll << 31)) return MERIT_ERR_INVALID_ARG;
            q.shape[i] = (int)o.shape[i];
            q.pitch[i] = elems;
            elems *= o.shape[i];
            if (elems >= (1ll << 40)) return MERIT_ERR_UNSUPPORTED;
        }
        // every coordinate any k can produce stays a small integer
        int64_t lo[MERIT_MAX_DIMS] = {0}, hi[MERIT_MAX_DIMS] = {0};
        for (int j = 0; j < nidx; ++j) {
            q.axis[j] = o.axis[j];
            if (o.stride[j] <= -INT_LIMIT || o.stride[j] >= INT_LIMIT || o.offset[j] <= -INT_LIMIT || o.offset[j] >= INT_LIMIT)
                return MERIT_ERR_UNSUPPORTED;
            q.stride[j] = (int)o.stride[j]; q.offset[j] = (int)o.offset[j];
            if (o.axis[j] < 0) continue;
            const int64_t travel = (d.range[j] > 0 ? d.range[j] - 1 : 0) * o.stride[j];
            lo[o.axis[j]] += o.offset[j] + (travel < 0 ? travel : 0);
            hi[o.axis[j]] += o.offset[j] + (travel > 0 ? travel : 0);
            if (lo[o.axis[j]] <= -INT_LIMIT || hi[o.axis[j]] >= INT_LIMIT) return MERIT_ERR_UNSUPPORTED;
        }
        return MERIT_OK;
    };
    if (merit_status st = operand(d.a, g.a); st != MERIT_OK) return st;
    if (g.mode == 0) {
        if (merit_status st = operand(d.b, g.b); st != MERIT_OK) return st;
    } else {
        for (int j = 0; j < MERIT_MAX_INDEX; ++j) g.b.axis[j] = -1;
    }
    pl->generic = 1;
    pl->out_ndim = d.n_par;
    for (int j = 0; j < d.n_par; ++j) pl->out_shape[j] = d.range[j];
    merit_launch_info &li = pl->info;
    std::memset(&li, 0, sizeof(li));
    li.kernel = generic_kernel_name(g);
    li.grid[0] = cdiv(rows, 256); li.grid[1] = 1; li.grid[2] = 1;
    li.block[0] = 256; li.block[1] = 1; li.block[2] = 1;
    li.lds_bytes = 0;
    // a workgroup: 256 consecutive rows (the last parallel index fastest), the whole accumulation range
    for (int j = 0; j < nidx; ++j) li.tile[j] = j < d.n_par ? 1 : d.range[j];
    li.tile[d.n_par - 1] = d.range[d.n_par - 1] < 256 ? d.range[d.n_par - 1] : 256;
    return MERIT_OK;
}

bool aligned16(const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) == 0; }

}  // namespace

// ============================================================== C ABI ======
extern "C" {

merit_status merit_plan_create(const merit_plan_desc *desc, merit_plan **out)
{
    if (!desc || !out) return MERIT_ERR_NULL;
    *out = nullptr;
    if ((int)desc->op < 0 || (int)desc->op > 12 || (int)desc->dtype < 0 || (int)desc->dtype > 2 ||
        (int)desc->pad < 0 || (int)desc->pad > 3)
        return MERIT_ERR_INVALID_ARG;
    if (desc->n_par < 1 || desc->n_acc < 1 || desc->n_par + desc->n_acc > MERIT_MAX_INDEX)
        return MERIT_ERR_INVALID_ARG;
    if (desc->a.ndim < 1 || desc->a.ndim > MERIT_MAX_DIMS || desc->b.ndim < 0 || desc->b.ndim > MERIT_MAX_DIMS)
        return MERIT_ERR_INVALID_ARG;
    const int nidx = desc->n_par + desc->n_acc;
    for (int j = 0; j < nidx; ++j) {
        if (desc->range[j] < 0) return MERIT_ERR_INVALID_ARG;
        if (desc->a.axis[j] < MERIT_AXIS_UNUSED || desc->a.axis[j] >= desc->a.ndim) return MERIT_ERR_INVALID_ARG;
        if (desc->b.ndim > 0 && (desc->b.axis[j] < MERIT_AXIS_UNUSED || desc->b.axis[j] >= desc->b.ndim))
            return MERIT_ERR_INVALID_ARG;
    }
    merit_plan *pl = new (std::nothrow) merit_plan;
    if (!pl) return MERIT_ERR_INVALID_ARG;
    std::memset(pl, 0, sizeof(*pl));
    pl->desc = *desc;
    merit_status st;
    switch (desc->op) {
    case MERIT_OP_CONV_DOT:
    case MERIT_OP_CONV_DOT_RELU:
    case MERIT_OP_CONV_DOT_POOLMAX:
    case MERIT_OP_CONV_DOT_RELU_POOLMAX:
    case MERIT_OP_CONV_DOT_ADD:
    case MERIT_OP_CONV_DOT_ADD_RELU: st = derive_conv(pl); break;
    case MERIT_OP_POOL_MAX:
    case MERIT_OP_POOL_AVG: st = derive_pool(pl); break;
    case MERIT_OP_CORR_DOT: st = derive_corr(pl); break;
    case MERIT_OP_DWCONV_DOT: st = derive_dw(pl); break;
    case MERIT_OP_SEPFILTER_DOT: st = derive_sep(pl); break;
    case MERIT_OP_BILATERAL: st = derive_bilateral(pl); break;
    default: st = derive_sad(pl); break;
    }
    // no specialised kernel for this descriptor: the definition kernel takes what it can
    if (st == MERIT_ERR_UNSUPPORTED) {
        const merit_status sg = derive_generic(pl);
        if (sg != MERIT_ERR_UNSUPPORTED) st = sg;
    }
    if (st != MERIT_OK) {
        delete pl;
        return st;
    }
    *out = pl;
    return MERIT_OK;
}

merit_status merit_plan_destroy(merit_plan *plan)
{
    if (!plan) return MERIT_ERR_NULL;
    delete plan;
    return MERIT_OK;
}

}  // extern "C"

static merit_status plan_conv2d_op(merit_op op, int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh,
                                   int sw, int ph, int pw, int dh, int dw, merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (N < 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 ||
        ph < 0 || pw < 0 || dh <= 0 || dw <= 0)
        return MERIT_ERR_INVALID_ARG;
    const int64_t eh = ((int64_t)kh - 1) * dh + 1, ew = ((int64_t)kw - 1) * dw + 1;
    if (H + 2 * ph < eh || W + 2 * pw < ew) return MERIT_ERR_SHAPE;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = op; d.dtype = MERIT_F16; d.pad = MERIT_PAD_ZERO;
    d.n_par = 4; d.n_acc = 3;
    const int64_t OH = out_extent(H, eh, sh, ph), OW = out_extent(W, ew, sw, pw);
    const int64_t range[7] = {N, Cout, OH, OW, Cin, kh, kw};
    const int ax[7] = {0, MERIT_AXIS_UNUSED, 2, 3, 1, 2, 3};
    const int64_t sx[7] = {1, 0, sh, sw, 1, dh, dw};
    const int64_t ox[7] = {0, 0, 0, 0, 0, -ph, -pw};
    const int aw[7] = {MERIT_AXIS_UNUSED, 0, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1, 2, 3};
    const int64_t sw_[7] = {0, 1, 0, 0, 1, 1, 1};
    for (int j = 0; j < 7; ++j) {
        d.range[j] = range[j];
        d.a.axis[j] = ax[j]; d.a.stride[j] = sx[j]; d.a.offset[j] = ox[j];
        d.b.axis[j] = aw[j]; d.b.stride[j] = sw_[j]; d.b.offset[j] = 0;
    }
    d.a.ndim = 4; d.a.shape[0] = N; d.a.shape[1] = Cin; d.a.shape[2] = H; d.a.shape[3] = W;
    d.b.ndim = 4; d.b.shape[0] = Cout; d.b.shape[1] = Cin; d.b.shape[2] = kh; d.b.shape[3] = kw;
    return merit_plan_create(&d, out);
}

extern "C" {

merit_status merit_plan_conv2d(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw,
                               int ph, int pw, merit_plan **out)
{
    return plan_conv2d_op(MERIT_OP_CONV_DOT, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, out);
}

merit_status merit_plan_conv2d_relu(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw,
                                    int ph, int pw, merit_plan **out)
{
    return plan_conv2d_op(MERIT_OP_CONV_DOT_RELU, N, Cin, H, W, Cout, kh, kw, sh, sw, ph, pw, 1, 1, out);
}

merit_status merit_plan_conv2d_dilated(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw,
                                       int ph, int pw, int dh, int dw, int relu, merit_plan **out)
{
    return plan_conv2d_op(relu ? MERIT_OP_CONV_DOT_RELU : MERIT_OP_CONV_DOT, N, Cin, H, W, Cout, kh, kw, sh, sw, ph,
                          pw, dh, dw, out);
}

merit_status merit_plan_conv2d_pool(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw,
                                    int ph, int pw, int relu, merit_plan **out)
{
    return plan_conv2d_op(relu ? MERIT_OP_CONV_DOT_RELU_POOLMAX : MERIT_OP_CONV_DOT_POOLMAX, N, Cin, H, W, Cout,
                          kh, kw, sh, sw, ph, pw, 1, 1, out);
}

merit_status merit_plan_conv2d_residual(int N, int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw,
                                        int ph, int pw, int relu, merit_plan **out)
{
    return plan_conv2d_op(relu ? MERIT_OP_CONV_DOT_ADD_RELU : MERIT_OP_CONV_DOT_ADD, N, Cin, H, W, Cout, kh, kw, sh,
                          sw, ph, pw, 1, 1, out);
}

merit_status merit_plan_pool2d(int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                               int is_avg, merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
        return MERIT_ERR_INVALID_ARG;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return MERIT_ERR_SHAPE;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = is_avg ? MERIT_OP_POOL_AVG : MERIT_OP_POOL_MAX;
    d.dtype = MERIT_F32;
    d.pad = is_avg ? MERIT_PAD_EXCLUDE : MERIT_PAD_NEG_INF;
    d.n_par = 4; d.n_acc = 2;
    const int64_t OH = out_extent(H, kh, sh, ph), OW = out_extent(W, kw, sw, pw);
    const int64_t range[6] = {N, C, OH, OW, kh, kw};
    const int ax[6] = {0, 1, 2, 3, 2, 3};
    const int64_t sx[6] = {1, 1, sh, sw, 1, 1};
    const int64_t ox[6] = {0, 0, 0, 0, -ph, -pw};
    for (int j = 0; j < 6; ++j) {
        d.range[j] = range[j];
        d.a.axis[j] = ax[j]; d.a.stride[j] = sx[j]; d.a.offset[j] = ox[j];
    }
    d.a.ndim = 4; d.a.shape[0] = N; d.a.shape[1] = C; d.a.shape[2] = H; d.a.shape[3] = W;
    d.b.ndim = 0;
    return merit_plan_create(&d, out);
}

static merit_status plan_window_filter(merit_op op, int N, int H, int W, int k, merit_plan **out);

merit_status merit_plan_sepfilter(int N, int H, int W, int k, merit_plan **out)
{
    return plan_window_filter(MERIT_OP_SEPFILTER_DOT, N, H, W, k, out);
}

merit_status merit_plan_bilateral(int N, int H, int W, int k, merit_plan **out)
{
    return plan_window_filter(MERIT_OP_BILATERAL, N, H, W, k, out);
}

merit_status merit_bilateral(const merit_plan *plan, const void *x, const void *gx, const void *gy, double norm,
                             void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_BILATERAL) return MERIT_ERR_INVALID_ARG;
    if (!(norm == norm) || norm * 1.4426950408889634 > 3.0e38 || norm * 1.4426950408889634 < -3.0e38)
        return MERIT_ERR_INVALID_ARG;
    if (plan->bil.N == 0) return MERIT_OK;                // empty batch: nothing to read or write
    if (!x || !gx || !gy || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(y) || ((uintptr_t)gx & 3) || ((uintptr_t)gy & 3)) return MERIT_ERR_ALIGNMENT;
    merit::BilatParams p = plan->bil;                     // the plan stays shareable between threads
    p.neg = norm <= 0.0 ? 1 : 0;
    p.scale = (float)std::sqrt(std::fabs(norm) * 1.4426950408889634);
    return launch_bilateral(p, static_cast<const float *>(x), static_cast<const float *>(gx),
                            static_cast<const float *>(gy), static_cast<float *>(y),
                            static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

}  // extern "C"

// k = (n, p1, p2 | a1, a2): the image window at offset -k/2 on both axes, a vector of length k on a2
static merit_status plan_window_filter(merit_op op, int N, int H, int W, int k, merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (N < 0 || H <= 0 || W <= 0 || k <= 0) return MERIT_ERR_INVALID_ARG;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = op; d.dtype = MERIT_F32; d.pad = MERIT_PAD_CLAMP;
    d.n_par = 3; d.n_acc = 2;
    const int64_t range[5] = {N, H, W, k, k};
    const int ax[5] = {0, 1, 2, 1, 2};
    const int64_t ox[5] = {0, 0, 0, -(int64_t)(k / 2), -(int64_t)(k / 2)};
    for (int j = 0; j < 5; ++j) {
        d.range[j] = range[j];
        d.a.axis[j] = ax[j]; d.a.stride[j] = 1; d.a.offset[j] = ox[j];
        d.b.axis[j] = j == 4 ? 0 : MERIT_AXIS_UNUSED; d.b.stride[j] = j == 4 ? 1 : 0; d.b.offset[j] = 0;
    }
    d.a.ndim = 3; d.a.shape[0] = N; d.a.shape[1] = H; d.a.shape[2] = W;
    d.b.ndim = 1; d.b.shape[0] = k;
    return merit_plan_create(&d, out);
}

// The stream-ordered temporaries of the two-launch plans come from the device's default memory
// pool.  By default that pool hands freed memory back to the system at the next synchronisation,
// so a caller who synchronises between calls would pay a device allocation per call (measured: 79
// against 69 us per call for the one-kernel form, which is slower on the GPU).  Once per device the
// pool's release threshold is raised so that it keeps what it has been given.
static void keep_pool_memory_once()
{
    static std::atomic<int> done[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return;
    if (done[dev].load(std::memory_order_acquire)) return;
    hipMemPool_t pool = nullptr;
    if (hipDeviceGetDefaultMemPool(&pool, dev) == hipSuccess && pool) {
        uint64_t keep = UINT64_MAX;
        (void)hipMemPoolSetAttribute(pool, hipMemPoolAttrReleaseThreshold, &keep);
    }
    done[dev].store(1, std::memory_order_release);
}

extern "C" {

merit_status merit_sepfilter(const merit_plan *plan, const void *x, const void *kx, const void *ky, void *y,
                             void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_SEPFILTER_DOT) return MERIT_ERR_INVALID_ARG;
    if (plan->sep.N == 0) return MERIT_OK;                // empty batch: nothing to read or write
    if (!x || !kx || !ky || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(y) || ((uintptr_t)kx & 3) || ((uintptr_t)ky & 3)) return MERIT_ERR_ALIGNMENT;
    return launch_sepfilter(plan->sep, static_cast<const float *>(x), static_cast<const float *>(kx),
                            static_cast<const float *>(ky), static_cast<float *>(y),
                            static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_plan_sad(int H, int W, int block, int range, merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (H <= 0 || W <= 0 || block <= 0 || range < 0) return MERIT_ERR_INVALID_ARG;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = MERIT_OP_SAD_ARGMIN; d.dtype = MERIT_U8; d.pad = MERIT_PAD_CLAMP;
    d.n_par = 2; d.n_acc = 4;
    const int64_t n = 2 * (int64_t)range + 1;
    const int64_t rg[6] = {cdiv(H, block), cdiv(W, block), n, n, block, block};
    const int a_ref[6] = {0, 1, 0, 1, 0, 1};
    const int64_t s_ref[6] = {block, block, 1, 1, 1, 1};
    const int64_t o_ref[6] = {0, 0, -range, -range, 0, 0};
    const int a_cur[6] = {0, 1, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 0, 1};
    const int64_t s_cur[6] = {block, block, 0, 0, 1, 1};
    for (int j = 0; j < 6; ++j) {
        d.range[j] = rg[j];
        d.a.axis[j] = a_ref[j]; d.a.stride[j] = s_ref[j]; d.a.offset[j] = o_ref[j];
        d.b.axis[j] = a_cur[j]; d.b.stride[j] = s_cur[j]; d.b.offset[j] = 0;
    }
    d.a.ndim = 2; d.a.shape[0] = H; d.a.shape[1] = W;
    d.b.ndim = 2; d.b.shape[0] = H; d.b.shape[1] = W;
    return merit_plan_create(&d, out);
}

merit_status merit_plan_set_tile(merit_plan *plan, const int64_t tile[MERIT_MAX_INDEX])
{
    if (!plan || !tile) return MERIT_ERR_NULL;
    if (plan->generic) {                                   // the definition kernel has one shape: nothing to choose
        for (int j = 0; j < MERIT_MAX_INDEX; ++j)
            if (tile[j] > 0) return MERIT_ERR_UNSUPPORTED;
        return MERIT_OK;
    }
    merit_plan trial = *plan;
    for (int j = 0; j < MERIT_MAX_INDEX; ++j) trial.tile_req[j] = tile[j];
    merit_status st;
    switch (trial.desc.op) {
    case MERIT_OP_CONV_DOT:
    case MERIT_OP_CONV_DOT_RELU:
    case MERIT_OP_CONV_DOT_POOLMAX:
    case MERIT_OP_CONV_DOT_RELU_POOLMAX:
    case MERIT_OP_CONV_DOT_ADD:
    case MERIT_OP_CONV_DOT_ADD_RELU: st = derive_conv(&trial); break;
    case MERIT_OP_POOL_MAX:
    case MERIT_OP_POOL_AVG: st = derive_pool(&trial); break;
    case MERIT_OP_CORR_DOT: st = derive_corr(&trial); break;
    case MERIT_OP_DWCONV_DOT: st = derive_dw(&trial); break;
    case MERIT_OP_SEPFILTER_DOT: st = derive_sep(&trial); break;
    case MERIT_OP_BILATERAL: st = derive_bilateral(&trial); break;
    default: st = derive_sad(&trial); break;
    }
    if (st != MERIT_OK) return st;          // the plan keeps its previous tiling
    *plan = trial;
    return MERIT_OK;
}

merit_status merit_plan_get_desc(const merit_plan *plan, merit_plan_desc *out)
{
    if (!plan || !out) return MERIT_ERR_NULL;
    *out = plan->desc;
    return MERIT_OK;
}

merit_status merit_plan_out_shape(const merit_plan *plan, int32_t *ndim, int64_t shape[MERIT_MAX_DIMS])
{
    if (!plan || !ndim || !shape) return MERIT_ERR_NULL;
    *ndim = plan->out_ndim;
    for (int i = 0; i < MERIT_MAX_DIMS; ++i) shape[i] = i < plan->out_ndim ? plan->out_shape[i] : 0;
    return MERIT_OK;
}

merit_status merit_plan_footprint(const merit_plan *plan, int which, const int64_t tile[MERIT_MAX_INDEX],
                                  int64_t out[MERIT_MAX_DIMS])
{
    if (!plan || !tile || !out) return MERIT_ERR_NULL;
    if (which != 0 && which != 1) return MERIT_ERR_INVALID_ARG;
    const merit_operand &o = which == 0 ? plan->desc.a : plan->desc.b;
    if (o.ndim == 0) return MERIT_ERR_INVALID_ARG;
    const int nidx = plan->desc.n_par + plan->desc.n_acc;
    for (int j = 0; j < nidx; ++j)
        if (tile[j] < 1 || tile[j] > plan->desc.range[j]) return MERIT_ERR_INVALID_ARG;
    for (int i = 0; i < MERIT_MAX_DIMS; ++i) {
        int64_t n = 0;
        if (i < o.ndim) {
            n = 1;
            for (int j = 0; j < nidx; ++j)
                if (o.axis[j] == i) n += (tile[j] - 1) * o.stride[j];
        }
        out[i] = n;
    }
    return MERIT_OK;
}

merit_status merit_plan_launch_info(const merit_plan *plan, merit_launch_info *out)
{
    if (!plan || !out) return MERIT_ERR_NULL;
    *out = plan->info;
    return MERIT_OK;
}

// a plan on the definition kernel: the same pointer rules as everywhere
static merit_status run_generic(const merit_plan *plan, const void *a, const void *b, void *y, void *stream)
{
    if (plan->gen.rows == 0) return MERIT_OK;             // an empty parallel range: nothing to read or write
    if (!a || !b || !y) return MERIT_ERR_NULL;
    if (!aligned16(a) || !aligned16(b) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_generic(plan->gen, a, b, y, static_cast<hipStream_t>(stream)) == hipSuccess ? MERIT_OK : MERIT_ERR_HIP;
}

merit_status merit_conv2d(const merit_plan *plan, const void *x, const void *w, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_CONV_DOT && plan->desc.op != MERIT_OP_CONV_DOT_RELU &&
        plan->desc.op != MERIT_OP_CONV_DOT_POOLMAX && plan->desc.op != MERIT_OP_CONV_DOT_RELU_POOLMAX)
        return MERIT_ERR_INVALID_ARG;
    if (plan->generic) return run_generic(plan, x, w, y, stream);
    if (plan->conv.N == 0) return MERIT_OK;               // empty batch: nothing to read or write
    if (!x || !w || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    if (plan->two_pass) {
        // the plain convolution into the plan's buffer on this device, then the pooling kernel
        // The convolution's result lives in a stream-ordered temporary: allocated and released in
        // the caller's stream, so calls on different streams never share it and the plan stays
        // immutable.  (The pool that serves it keeps the memory for the next call.)
        const ConvParams &q = plan->conv2;
        hipStream_t s = static_cast<hipStream_t>(stream);
        keep_pool_memory_once();
        void *mid = nullptr;
        if (hipMallocAsync(&mid, (size_t)q.N * q.Cout * q.OH * q.OW * 2, s) != hipSuccess || !mid) return MERIT_ERR_HIP;
        hipError_t e = launch_conv2d(q, x, w, nullptr, mid, s);
        if (e == hipSuccess) e = launch_maxpool_f16(mid, y, (int64_t)q.N * q.Cout, q.OH, q.OW, s);
        const hipError_t ef = hipFreeAsync(mid, s);
        return (e == hipSuccess && ef == hipSuccess) ? MERIT_OK : MERIT_ERR_HIP;
    }
    return launch_conv2d(plan->conv, x, w, nullptr, y, static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

static bool plan_takes_packed(const merit_plan *plan)
{
    return (plan->desc.op == MERIT_OP_CONV_DOT || plan->desc.op == MERIT_OP_CONV_DOT_RELU) &&
           plan->conv.variant == CONV_CHWS;
}

merit_status merit_plan_packed_weights_bytes(const merit_plan *plan, int64_t *bytes)
{
    if (!plan || !bytes) return MERIT_ERR_NULL;
    if (!plan_takes_packed(plan)) return MERIT_ERR_UNSUPPORTED;
    const ConvParams &p = plan->conv;
    *bytes = (int64_t)p.co_groups * p.nchunks * p.lds_w_bytes;
    return MERIT_OK;
}

merit_status merit_conv2d_pack_weights(const merit_plan *plan, const void *w, void *packed, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (!plan_takes_packed(plan)) return MERIT_ERR_UNSUPPORTED;
    if (!w || !packed) return MERIT_ERR_NULL;
    if (!aligned16(w) || !aligned16(packed)) return MERIT_ERR_ALIGNMENT;
    return launch_conv2d_pack_weights(plan->conv, w, packed, static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_conv2d_packed(const merit_plan *plan, const void *x, const void *packed, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (!plan_takes_packed(plan)) return MERIT_ERR_UNSUPPORTED;
    if (plan->conv.N == 0) return MERIT_OK;               // empty batch: nothing to read or write
    if (!x || !packed || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(packed) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_conv2d_chws(plan->conv, x, packed, nullptr, y, static_cast<hipStream_t>(stream), true) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_conv2d_packed_noalloc(const merit_plan *plan, const void *x, const void *w, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (!plan_takes_packed(plan)) return MERIT_ERR_UNSUPPORTED;
    const ConvParams &p = plan->conv;
    if ((int64_t)p.co_groups * p.nchunks * p.lds_w_bytes > (int64_t)MERIT_NOALLOC_SCRATCH_BYTES)
        return MERIT_ERR_SCRATCH_LIMIT;
    if (p.N == 0) return MERIT_OK;                        // empty batch: nothing to read or write
    if (!x || !w || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_conv2d_chws_noalloc(p, x, w, y, static_cast<hipStream_t>(stream)) == hipSuccess ? MERIT_OK
                                                                                                   : MERIT_ERR_HIP;
}

merit_status merit_conv2d_residual(const merit_plan *plan, const void *x, const void *w, const void *r, void *y,
                                   void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_CONV_DOT_ADD && plan->desc.op != MERIT_OP_CONV_DOT_ADD_RELU)
        return MERIT_ERR_INVALID_ARG;
    if (plan->conv.N == 0) return MERIT_OK;               // empty batch: nothing to read or write
    if (!x || !w || !r || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(r) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_conv2d(plan->conv, x, w, r, y, static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_pool2d(const merit_plan *plan, const void *x, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_POOL_MAX && plan->desc.op != MERIT_OP_POOL_AVG) return MERIT_ERR_INVALID_ARG;
    if (plan->generic) return run_generic(plan, x, x, y, stream);
    if (plan->pool.NC == 0) return MERIT_OK;              // empty batch: nothing to read or write
    if (!x || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_pool2d(plan->pool, static_cast<const float *>(x), static_cast<float *>(y),
                         static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_sad_search(const merit_plan *plan, const void *cur, const void *ref, void *sad, void *mv,
                              void *stream)
{
    if (!plan || !cur || !ref || !sad || !mv) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_SAD_ARGMIN) return MERIT_ERR_INVALID_ARG;
    if (!aligned16(cur) || !aligned16(ref) || !aligned16(sad) || !aligned16(mv)) return MERIT_ERR_ALIGNMENT;
    return launch_sad(plan->sad, static_cast<const uint8_t *>(cur), static_cast<const uint8_t *>(ref),
                      static_cast<int32_t *>(sad), static_cast<int32_t *>(mv),
                      static_cast<hipStream_t>(stream)) == hipSuccess
               ? MERIT_OK
               : MERIT_ERR_HIP;
}

merit_status merit_plan_conv2d_depthwise(int N, int C, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                                         merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || sh <= 0 || sw <= 0 || ph < 0 || pw < 0)
        return MERIT_ERR_INVALID_ARG;
    if (H + 2 * ph < kh || W + 2 * pw < kw) return MERIT_ERR_SHAPE;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = MERIT_OP_DWCONV_DOT; d.dtype = MERIT_F16; d.pad = MERIT_PAD_ZERO;
    d.n_par = 4; d.n_acc = 2;
    const int64_t OH = out_extent(H, kh, sh, ph), OW = out_extent(W, kw, sw, pw);
    const int64_t range[6] = {N, C, OH, OW, kh, kw};
    const int ax[6] = {0, 1, 2, 3, 2, 3};
    const int64_t sx[6] = {1, 1, sh, sw, 1, 1};
    const int64_t ox[6] = {0, 0, 0, 0, -ph, -pw};
    const int aw[6] = {MERIT_AXIS_UNUSED, 0, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1, 2};
    const int64_t sw_[6] = {0, 1, 0, 0, 1, 1};
    for (int j = 0; j < 6; ++j) {
        d.range[j] = range[j];
        d.a.axis[j] = ax[j]; d.a.stride[j] = sx[j]; d.a.offset[j] = ox[j];
        d.b.axis[j] = aw[j]; d.b.stride[j] = sw_[j]; d.b.offset[j] = 0;
    }
    d.a.ndim = 4; d.a.shape[0] = N; d.a.shape[1] = C; d.a.shape[2] = H; d.a.shape[3] = W;
    d.b.ndim = 3; d.b.shape[0] = C; d.b.shape[1] = kh; d.b.shape[2] = kw;
    return merit_plan_create(&d, out);
}

merit_status merit_conv2d_depthwise(const merit_plan *plan, const void *x, const void *w, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_DWCONV_DOT) return MERIT_ERR_INVALID_ARG;
    if (plan->generic) return run_generic(plan, x, w, y, stream);
    if (plan->dw.NC == 0) return MERIT_OK;                // empty batch: nothing to read or write
    if (!x || !w || !y) return MERIT_ERR_NULL;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_dwconv(plan->dw, x, w, y, static_cast<hipStream_t>(stream)) == hipSuccess ? MERIT_OK : MERIT_ERR_HIP;
}

merit_status merit_plan_correlation(int N, int C, int H, int W, int R, int sd, merit_plan **out)
{
    if (!out) return MERIT_ERR_NULL;
    *out = nullptr;
    if (N < 0 || C <= 0 || H <= 0 || W <= 0 || R < 0 || sd <= 0) return MERIT_ERR_INVALID_ARG;
    merit_plan_desc d;
    std::memset(&d, 0, sizeof(d));
    d.op = MERIT_OP_CORR_DOT; d.dtype = MERIT_F16; d.pad = MERIT_PAD_ZERO;
    d.n_par = 5; d.n_acc = 1;
    const int64_t n = 2 * (int64_t)R + 1;
    const int64_t range[6] = {N, H, W, n, n, C};
    const int a1[6] = {0, 2, 3, MERIT_AXIS_UNUSED, MERIT_AXIS_UNUSED, 1};
    const int64_t s1[6] = {1, 1, 1, 0, 0, 1};
    const int a2[6] = {0, 2, 3, 2, 3, 1};
    const int64_t s2[6] = {1, 1, 1, sd, sd, 1};
    const int64_t o2[6] = {0, 0, 0, -(int64_t)R * sd, -(int64_t)R * sd, 0};
    for (int j = 0; j < 6; ++j) {
        d.range[j] = range[j];
        d.a.axis[j] = a1[j]; d.a.stride[j] = s1[j]; d.a.offset[j] = 0;
        d.b.axis[j] = a2[j]; d.b.stride[j] = s2[j]; d.b.offset[j] = o2[j];
    }
    d.a.ndim = 4; d.a.shape[0] = N; d.a.shape[1] = C; d.a.shape[2] = H; d.a.shape[3] = W;
    d.b.ndim = 4; d.b.shape[0] = N; d.b.shape[1] = C; d.b.shape[2] = H; d.b.shape[3] = W;
    return merit_plan_create(&d, out);
}

merit_status merit_correlation(const merit_plan *plan, const void *x1, const void *x2, void *y, void *stream)
{
    if (!plan) return MERIT_ERR_NULL;
    if (plan->desc.op != MERIT_OP_CORR_DOT) return MERIT_ERR_INVALID_ARG;
    if (plan->generic) return run_generic(plan, x1, x2, y, stream);
    if (plan->corr.N == 0) return MERIT_OK;               // empty batch: nothing to read or write
    if (!x1 || !x2 || !y) return MERIT_ERR_NULL;
    if (!aligned16(x1) || !aligned16(x2) || !aligned16(y)) return MERIT_ERR_ALIGNMENT;
    return launch_correlation(plan->corr, x1, x2, y, static_cast<hipStream_t>(stream)) == hipSuccess ? MERIT_OK
                                                                                                   : MERIT_ERR_HIP;
}

const char *merit_status_string(merit_status s)
{
    switch ((int)s) {          // a C caller may pass any int
    case MERIT_OK: return "ok";
    case MERIT_ERR_NULL: return "null pointer";
    case MERIT_ERR_INVALID_ARG: return "invalid argument";
    case MERIT_ERR_SHAPE: return "inconsistent shape";
    case MERIT_ERR_UNSUPPORTED: return "transform not supported by any kernel";
    case MERIT_ERR_ALIGNMENT: return "device pointer not 16-byte aligned";
    case MERIT_ERR_HIP: return "HIP launch failed";
    case MERIT_ERR_SCRATCH_LIMIT: return "needs more scratch memory than the library's fixed buffer holds";
    }
    return "unknown status";
}

}  // extern "C"
