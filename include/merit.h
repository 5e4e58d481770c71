/*
 * merit.h -- C ABI of the MI355X (gfx950) ranged inner-product library.
 *
 * The library evaluates  Vec(C) = R(M(A), M(B), (.))  (paper Section III, Eq. 1):
 * every output element p reduces, with a product function (.), the row p of the
 * transformed tensors M(A), M(B), where
 *
 *     M(A)[p,a] = A[x],  x_i = sum_j delta(i, d_j) * (k_j * s_j + o_j),  k = (p,a)
 *                                                    (Section III-C, Eq. 5).
 *
 * M(.) is never stored: each kernel stages the minimal covering sub-tensor of a
 * tile (Section IV-A, Eq. 9) in LDS and expands it from there.
 *
 * Conventions for every entry point
 *   - Tensor pointers are DEVICE pointers owned by the caller, dense row-major,
 *     16-byte aligned (else MERIT_ERR_ALIGNMENT).  Nothing is copied or kept.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Work is enqueued and the call returns; the library never synchronises and
 *     never allocates device memory -- with one exception, a convolution +
 *     pooling plan that runs as two launches (see merit_plan_conv2d_pool), which
 *     takes a stream-ordered temporary (hipMallocAsync / hipFreeAsync in the
 *     caller's stream) and, at its first launch on a device, raises the release
 *     threshold of that device's default memory pool so that the pool keeps the
 *     memory across synchronisations.
 *   - A plan is immutable host memory; it may be shared between threads and
 *     streams.  Plans are created and destroyed without touching the GPU.
 *   - Every function returns a merit_status; on any error nothing was launched.
 *   - A plan whose output is empty (batch size 0) makes the operation a no-op
 *     that returns MERIT_OK without looking at the tensor pointers.
 */
#ifndef MERIT_H
#define MERIT_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MERIT_MAX_INDEX 12   /* |p| + |a| */
#define MERIT_MAX_DIMS  6

typedef enum {
    MERIT_OK = 0,
    MERIT_ERR_NULL,          /* a required pointer is NULL                         */
    MERIT_ERR_INVALID_ARG,   /* enum out of range, negative size, ...              */
    MERIT_ERR_SHAPE,         /* ranges/shapes inconsistent with each other         */
    MERIT_ERR_UNSUPPORTED,   /* a valid transform that no kernel here implements   */
    MERIT_ERR_ALIGNMENT,     /* device pointer not 16-byte aligned                 */
    MERIT_ERR_HIP,           /* the HIP runtime refused the launch                 */
    MERIT_ERR_SCRATCH_LIMIT  /* more scratch memory needed than the library's fixed buffer holds */
} merit_status;

/* Product functions (.) (Section III-B): dot product (Eq. 3); max / mean of the
 * window (one operand; the paper names pooling only as a max/min use, Table
 * "isa"); L1 distance (Eq. 4) followed by min/argmin over the leading
 * accumulation indices (the outer level of a 2-level ranged inner product);
 * the clipped dot product max(v1^T v2, 0), the fused ReLU layer (second
 * definition of (.) in Section III-B; PostLoop of Listing 1). */
typedef enum {
    MERIT_OP_CONV_DOT = 0,
    MERIT_OP_POOL_MAX = 1,
    MERIT_OP_POOL_AVG = 2,
    MERIT_OP_SAD_ARGMIN = 3,
    MERIT_OP_CONV_DOT_RELU = 4,
    MERIT_OP_CORR_DOT = 5,    /* dot product over channels of two displaced tensors (Eq. 8) */
    MERIT_OP_DWCONV_DOT = 6,  /* dot product over the window only: one kernel per channel   */
    /* convolution (plain / clipped product) whose binary16 result goes through a 3x3, stride 2,
     * padding 1 max pooling before it leaves the chip: the fused "CONV+Pool" layers of the
     * per-layer network table in Section VI-C.  The descriptor is the convolution's. */
    MERIT_OP_CONV_DOT_POOLMAX = 7,
    MERIT_OP_CONV_DOT_RELU_POOLMAX = 8,
    /* residual layer: a tensor of the output's shape is loaded and added to the accumulated sum
     * in PostLoop (Section III-B, the remark after Listing 1), then the optional clip, then the
     * one rounding.  The descriptor is the convolution's; the third tensor is an argument of
     * merit_conv2d_residual. */
    MERIT_OP_CONV_DOT_ADD = 9,
    MERIT_OP_CONV_DOT_ADD_RELU = 10,
    /* separable filter: a k x k window whose taps are the outer product of two vectors, run as
     * two 1-D dot-product passes (along the width, then along the height).  Descriptor:
     * k = (n, p1, p2 | a1, a2), a = the image [N,H,W] with the window indices on axes 1 and 2
     * at offset -k/2 (the bilateral-filter call of Section VI-A); b = the vector of length k
     * indexed by a2; the vector indexed by a1 is a further argument of merit_sepfilter. */
    MERIT_OP_SEPFILTER_DOT = 11,
    /* bilateral filter: the strategy class of Section VI-A (Listing 2) on the k x k window of
     * Listing 3; descriptor as for the separable filter (image window at offset -k/2, b = the
     * spatial lookup table indexed by a2; the table indexed by a1 and the range constant are
     * arguments of merit_bilateral) */
    MERIT_OP_BILATERAL = 12
} merit_op;

typedef enum { MERIT_U8 = 0, MERIT_F16 = 1, MERIT_F32 = 2 } merit_dtype;

/* What an out-of-range coordinate x yields. */
typedef enum {
    MERIT_PAD_ZERO = 0,      /* the value 0                      (CONV_DOT)        */
    MERIT_PAD_NEG_INF = 1,   /* -infinity                        (POOL_MAX)        */
    MERIT_PAD_EXCLUDE = 2,   /* not part of the reduction/count  (POOL_AVG)        */
    MERIT_PAD_CLAMP = 3      /* nearest in-range element         (SAD_ARGMIN)      */
} merit_pad;

#define MERIT_AXIS_UNUSED (-1)

/* One operand's transform: for every index k_j the axis d_j it moves along
 * (MERIT_AXIS_UNUSED if none), its stride s_j and offset o_j (Eq. 5). */
typedef struct {
    int32_t ndim;
    int64_t shape [MERIT_MAX_DIMS];
    int32_t axis  [MERIT_MAX_INDEX];
    int64_t stride[MERIT_MAX_INDEX];
    int64_t offset[MERIT_MAX_INDEX];
} merit_operand;

/* Plain data, caller-owned, copied by merit_plan_create.
 * range[] lists the extents of k = (p, a): n_par parallel indices first, then
 * n_acc accumulation indices (the NDRange of Section III-C, Eq. 6).
 *
 * Patterns with a specialised kernel
 *   CONV_DOT   F16 ZERO     k=(n,co,oy,ox | ci,ky,kx)  a = x[N,Cin,H,W], b = w[Cout,Cin,kh,kw]
 *   CONV_DOT_RELU           same
 *   POOL_MAX   F32 NEG_INF  k=(n,c,oy,ox | ky,kx)      a = x[N,C,H,W],   b unused (ndim 0)
 *   POOL_AVG   F32 EXCLUDE  same
 *   SAD_ARGMIN U8  CLAMP    k=(by,bx | dy,dx,i,j)      a = ref[H,W] (displaced by dy,dx),
 *                                                      b = cur[H,W]
 *   DWCONV_DOT F16 ZERO     k=(n,c,oy,ox | ky,kx)      a = x[N,C,H,W], b = w[C,kh,kw]
 *   CORR_DOT   F16 ZERO     k=(n,p1,p2,p3,p4 | c)      a = x1[N,C,H,W] at (p1,p2),
 *                                                      b = x2[N,C,H,W] at (p1+(p3-R)*sd, p2+(p4-R)*sd)
 * with output extents equal to floor((I + 2*pad - e)/s) + 1, e = (k-1)*d + 1.  The
 * strides d of the window indices ky, kx must be 1 for pooling; for the CONV ops they are
 * the dilation (Section III-C, the example after Eq. 6), up to 16.
 *
 * Any other descriptor of a dot product (CONV_DOT, CONV_DOT_RELU, DWCONV_DOT, CORR_DOT: F16,
 * padding ZERO or CLAMP, two operands) or of a single-operand reduction (POOL_MAX: F32, any
 * padding rule; POOL_AVG: F32, EXCLUDE, ZERO or CLAMP) runs on one kernel that evaluates Eq. 5
 * as it reads, a thread per row of M(A), M(B): any number of indices up to MERIT_MAX_INDEX with at
 * most MERIT_MAX_DIMS parallel ones, any axis, stride (negative too) and offset per index,
 * ranges of at least 1 for the accumulation indices.  Its output is the dense tensor of the
 * parallel ranges; it goes through the entry point of the descriptor's operation (merit_conv2d
 * for CONV_DOT / CONV_DOT_RELU with a = x, b = w).  launch_info().kernel names it
 * ("merit_generic<dot|max|mean>"); it takes no tile request.  Everything else is
 * MERIT_ERR_UNSUPPORTED. */
typedef struct {
    merit_op      op;
    merit_dtype   dtype;
    merit_pad     pad;
    int32_t       n_par, n_acc;
    int64_t       range[MERIT_MAX_INDEX];
    merit_operand a;
    merit_operand b;
} merit_plan_desc;

typedef struct merit_plan merit_plan;   /* opaque, host memory only */

/* Launch geometry a plan resolved to (for tests, profiling and roofline
 * accounting; informational). */
typedef struct {
    const char *kernel;      /* name of the HIP kernel the plan dispatches to      */
    int64_t grid[3];         /* workgroups                                         */
    int32_t block[3];        /* threads per workgroup                              */
    int64_t lds_bytes;       /* LDS per workgroup                                  */
    int64_t tile[MERIT_MAX_INDEX]; /* sub-tensor (t_p, t_a) one workgroup covers   */
} merit_launch_info;

/* ---- plans ---------------------------------------------------------------- */

/* Validate `desc` against the accepted patterns and derive output shape, tile
 * and halo geometry (Eq. 9) and grid.  *out receives a new plan (free it with
 * merit_plan_destroy).  Host only. */
merit_status merit_plan_create(const merit_plan_desc *desc, merit_plan **out);
merit_status merit_plan_destroy(merit_plan *plan);

/* Convenience constructors: fill the descriptor for the three 2-D operations
 * and call merit_plan_create.
 *  conv2d: y[n,co,oy,ox] = sum x[n,ci,oy*sh+ky-ph,ox*sw+kx-pw] * w[co,ci,ky,kx]
 *          (index pattern of Section III-C, Eq. 6: strided, no kernel flip).
 *          Any channel counts, window, stride and padding within the index limits: the
 *          planner picks an MFMA kernel (few input channels; all channels staged at once;
 *          channels in passes) and, where no MFMA layout holds the shape, a vector-ALU kernel
 *          (merit_launch_info.kernel names the choice).
 *  pool2d: max (is_avg=0) or mean over in-range elements (is_avg=1) of the window.
 *  sad:    frames [H,W] u8, ceil(H/block) x ceil(W/block) blocks of `block` x `block`
 *          pixels (blocks that reach past the frame edge read both frames with
 *          clamped coordinates, i.e. the border replicated),
 *          candidates dy,dx in [-range, range]; second tensor displaced by the
 *          search indices as in Section III-C, Eq. 8. */
merit_status merit_plan_conv2d(int N, int Cin, int H, int W, int Cout, int kh, int kw,
                               int sh, int sw, int ph, int pw, merit_plan **out);
/* The same transform with the product function max(v1^T v2, 0) (Section III-B):
 * y = max(sum, 0), clipped before the one rounding to binary16; never -0. */
merit_status merit_plan_conv2d_relu(int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                    int sh, int sw, int ph, int pw, merit_plan **out);
/* Dilated window: x[n,ci,oy*sh+ky*dh-ph,ox*sw+kx*dw-pw] (Section III-C, after Eq. 6);
 * relu != 0 selects the clipped product function. */
merit_status merit_plan_conv2d_dilated(int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                       int sh, int sw, int ph, int pw, int dh, int dw, int relu,
                                       merit_plan **out);
/* Convolution, optional clipping (relu != 0), then max pooling with a 3x3 window, stride 2,
 * padding 1 (-inf outside) of the binary16 convolution result, as one kernel: the convolution
 * output never reaches memory (the fused "CONV+Pool" layers of the per-layer table in
 * Section VI-C).  Output [N,Cout,OH/2,OW/2].  Two kernel families take it: few input
 * channels (Cin < 8, window rows of at most 8 taps, W % 8 == 0, OH even, OW % 16 == 0, OW <= 128)
 * and 3x3 windows on many (Cin % 8 == 0, Cin >= 16, Cout >= 33, OH and OW even, OW <= 128);
 * anything else is MERIT_ERR_UNSUPPORTED (run the two operations one after the other).
 * On many channels the planner compares two forms.  One kernel: work items are bands of pooled
 * rows, and every band below an image's first recomputes the convolution rows above it, which
 * a compute-bound layer on few images cannot hide (256 -> 256 channels on 56x56, 8 images: 1.8
 * times the plain convolution).  Two launches: the plain convolution into a temporary of its
 * result's size, taken from and returned to the stream's memory pool inside the call, then a
 * binary16 pooling kernel over it (the same values: maxima are exact).  merit_plan_launch_info
 * names the form ("merit_conv2d_chws_pool" or "merit_conv2d_chws+merit_maxpool_f16"); a tile
 * request (merit_plan_set_tile: 8 x 64, 8 x 32, 12 x 64) always selects the one-kernel form. */
merit_status merit_plan_conv2d_pool(int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                    int sh, int sw, int ph, int pw, int relu, merit_plan **out);
/* Residual layer (Section III-B, remark after Listing 1): y = x (*) w + r, or
 * max(x (*) w + r, 0) when relu != 0; r has the output's shape.  Run with
 * merit_conv2d_residual. */
merit_status merit_plan_conv2d_residual(int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                        int sh, int sw, int ph, int pw, int relu, merit_plan **out);
merit_status merit_plan_pool2d(int N, int C, int H, int W, int kh, int kw,
                               int sh, int sw, int ph, int pw, int is_avg, merit_plan **out);
/* Separable filter (a row of the paper's GPU speed-up table, Section VI-B) on N images of
 * H x W fp32 pixels with two tap vectors of length k <= 32:
 *   y[n,p1,p2] = sum_{a1,a2<k} ky[a1] kx[a2] x[n, p1 + a1 - k/2, p2 + a2 - k/2],
 * taps not flipped, coordinates clamped to the image (border replicated). */
merit_status merit_plan_sepfilter(int N, int H, int W, int k, merit_plan **out);
/* Bilateral filter (Section VI-A, Listings 2 and 3) on N images of H x W fp32 pixels, window
 * k x k (k <= 32) at offset -k/2, coordinates clamped to the image:
 *   y = sum w v / sum w,  w = exp((center - v)^2 * norm) * gy[a1] * gx[a2]. */
merit_status merit_plan_bilateral(int N, int H, int W, int k, merit_plan **out);
merit_status merit_plan_sad(int H, int W, int block, int range, merit_plan **out);
/* Depthwise convolution (the depthwise row of the paper's table of further workloads):
 * y[n,c,oy,ox] = sum_{ky,kx} x[n,c,oy*sh+ky-ph,ox*sw+kx-pw] * w[c,ky,kx]. */
merit_status merit_plan_conv2d_depthwise(int N, int C, int H, int W, int kh, int kw, int sh, int sw,
                                         int ph, int pw, merit_plan **out);
/* Correlation layer (Section III-C, Eq. 8): y[n,p1,p2,p3,p4] = sum_c x1[n,c,p1,p2] *
 * x2[n,c,p1+(p3-R)*sd,p2+(p4-R)*sd], p3,p4 in [0, 2R]; 0 outside the image; no
 * normalisation by the channel count.  W must be a multiple of 8, R <= 15, sd <= 8. */
merit_status merit_plan_correlation(int N, int C, int H, int W, int R, int sd, merit_plan **out);

/* Copy of the descriptor the plan was created from. */
merit_status merit_plan_get_desc(const merit_plan *plan, merit_plan_desc *out);
/* Output tensor shape: the parallel ranges ([N,Cout,OH,OW], [N,C,OH,OW], [nby,nbx],
 * [N,H,W,2R+1,2R+1]); [N,Cout,OH/2,OW/2] for a fused convolution + pooling plan. */
merit_status merit_plan_out_shape(const merit_plan *plan, int32_t *ndim, int64_t shape[MERIT_MAX_DIMS]);
/* Size of the minimal sub-tensor of operand `which` (0 = a, 1 = b) that contains
 * a tile of M(.) with extents tile[0 .. n_par+n_acc-1]:
 * 1 + sum_j (t_j - 1) s_j delta(d_j, i) per axis i  (Section IV-A, Eq. 9). */
merit_status merit_plan_footprint(const merit_plan *plan, int which,
                                  const int64_t tile[MERIT_MAX_INDEX], int64_t out[MERIT_MAX_DIMS]);
merit_status merit_plan_launch_info(const merit_plan *plan, merit_launch_info *out);
/* Override the sub-tensor (t_p, t_a) one workgroup covers; the paper's call
 * passes tile sizes next to the ranges (Section VI-A, Listing 3).  Entries <= 0
 * keep the library's choice.  Honoured entries: pooling tile[2] = output rows
 * (and tile[3] = output columns when the generic kernel is used); convolution
 * tile[2] = wavefronts per workgroup and tile[3] = consecutive output pixels per
 * multiplying wavefront.  4 x 32, 4 x 64 and (fewer than 8 input channels) 8 x 32:
 * every wavefront stages, multiplies and stores, tile[2]*tile[3] pixels per
 * workgroup.  8 x 64: 4 multiplying + 4 data-moving wavefronts, 256 pixels per
 * workgroup (x 64 output channels).  On 8 and more input channels (3x3, 1x1 and --
 * 8 x 64 only -- 5x5 windows, Cin % 8 == 0) also 8 x 128 (256 pixels x 128 channels), 8 x 32 (128
 * pixels x 64 channels, 32 input channels per pass) and 12 x 64 (8 multiplying +
 * 4 moving wavefronts, 256 pixels x 128 channels); a fused-pooling plan on many
 * channels takes 8 x 64, 8 x 32 and 12 x 64.  Block matching
 * tile[1] = blocks per workgroup (1, 4 or 8; a value the shape has no kernel for
 * keeps the library's choice); separable filter tile[1] = staged rows per workgroup
 * at most (output rows = that minus k - 1, rounded down to a multiple of 4).  On error
 * the plan is unchanged.  Not safe to
 * call while another thread launches with the same plan. */
merit_status merit_plan_set_tile(merit_plan *plan, const int64_t tile[MERIT_MAX_INDEX]);

/* ---- operations ------------------------------------------------------------
 * x_f16: [N,Cin,H,W] binary16; w_f16: [Cout,Cin,kh,kw] binary16;
 * y_f16: [N,Cout,OH,OW] binary16.  Products accumulate in fp32 on the matrix
 * cores and are rounded once (nearest even) to binary16.  (.) = Eq. 3, or its
 * clipped form for a CONV_DOT_RELU plan.  For a plan from merit_plan_conv2d_pool
 * y_f16 is the pooled tensor [N,Cout,OH/2,OW/2]: the exact maximum of the rounded
 * convolution results in each window. */
merit_status merit_conv2d(const merit_plan *plan, const void *x_f16, const void *w_f16,
                          void *y_f16, void *hip_stream);

/* Weights in pass order.  The kernel for layers with many input channels takes the channels
 * through LDS in passes (Section IV-A: one covering sub-tensor at a time) and needs, per pass,
 * each output channel's taps regrouped by eight input channels.  From the caller's
 * [Cout,Cin,kh,kw] tensor that is a register transposition on every pass of every tile; weights
 * do not change between calls, so the regrouping can be done once instead:
 *   merit_plan_packed_weights_bytes  size of the packed copy for this plan (a multiple of 16);
 *                                    MERIT_ERR_UNSUPPORTED if the plan's kernel takes no packed
 *                                    weights (merit_launch_info.kernel != "merit_conv2d_chws")
 *   merit_conv2d_pack_weights        w_f16 -> packed (device memory of that size, owned by the
 *                                    caller, 16-byte aligned); enqueued on the stream
 *   merit_conv2d_packed              merit_conv2d with the packed copy in place of w_f16; same
 *                                    result bit for bit.  The packed copy belongs to the plan's
 *                                    shape and tile: use it only with plans of that shape.
 * The library still owns no device memory. */
merit_status merit_plan_packed_weights_bytes(const merit_plan *plan, int64_t *bytes);
merit_status merit_conv2d_pack_weights(const merit_plan *plan, const void *w_f16, void *packed,
                                       void *hip_stream);
merit_status merit_conv2d_packed(const merit_plan *plan, const void *x_f16, const void *packed,
                                 void *y_f16, void *hip_stream);

/* For callers that cannot allocate device memory -- code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc: merit_conv2d_pack_weights and
 * merit_conv2d_packed in one call, with the packed copy in a fixed device buffer that lives
 * inside the library instead of one the caller brings.  The buffer is
 * MERIT_NOALLOC_SCRATCH_BYTES per GPU, part of the loaded library on every GPU it runs on
 * until the process ends; a plan whose packed weights are larger is refused with
 * MERIT_ERR_SCRATCH_LIMIT (nothing launched), a plan whose kernel takes no packed weights with
 * MERIT_ERR_UNSUPPORTED.  Neither this call nor anything it runs allocates or frees memory.
 * Every call on a GPU uses that GPU's one buffer and overwrites all of the part it needs:
 * two calls that overlap in time on one GPU (different streams, different threads) race and
 * give undefined results; calls on one stream are ordered and safe.  Same result, bit for
 * bit, as merit_conv2d_packed. */
#define MERIT_NOALLOC_SCRATCH_BYTES (8 << 20)
merit_status merit_conv2d_packed_noalloc(const merit_plan *plan, const void *x_f16, const void *w_f16,
                                         void *y_f16, void *hip_stream);

/* Residual layer: as merit_conv2d, with r_f16 [N,Cout,OH,OW] binary16 added to the fp32 sums
 * before the clip (if the plan has one) and the one rounding to binary16.  r_f16 may be
 * y_f16 itself (every element is read before it is overwritten, by the workgroup that owns
 * it); any other overlap of y with x, w or r is undefined.  The plan must come from
 * merit_plan_conv2d_residual (or a CONV_DOT_ADD / CONV_DOT_ADD_RELU descriptor). */
merit_status merit_conv2d_residual(const merit_plan *plan, const void *x_f16, const void *w_f16,
                                   const void *r_f16, void *y_f16, void *hip_stream);

/* x_f32: [N,C,H,W]; y_f32: [N,C,OH,OW].  max: exact.  avg: fp32 sum in window
 * scan order divided by the in-range count. */
merit_status merit_pool2d(const merit_plan *plan, const void *x_f32, void *y_f32, void *hip_stream);

/* x_f32, y_f32: [N,H,W]; kx_f32 (taps along the width), ky_f32 (along the height): [k], device
 * memory.  fp32 multiply-adds in tap order, the row pass first; its result stays on chip in
 * fp32.  y must not overlap x. */
merit_status merit_sepfilter(const merit_plan *plan, const void *x_f32, const void *kx_f32,
                             const void *ky_f32, void *y_f32, void *hip_stream);

/* x_f32, y_f32: [N,H,W]; gx_f32, gy_f32: the spatial lookup tables [k] (device memory), all
 * entries > 0; norm: the range constant of the strategy class (-1/(2 sigma_r^2) for a Gaussian
 * range term), passed by value like the listing's Constant.  fp32 arithmetic, the exponential
 * as 2^(d*d*norm*log2 e) with the hardware's base-2 exponential.  y must not overlap x. */
merit_status merit_bilateral(const merit_plan *plan, const void *x_f32, const void *gx_f32,
                             const void *gy_f32, double norm, void *y_f32, void *hip_stream);

/* cur_u8, ref_u8: [H,W] frames.  sad_i32: [nby*nbx] minimum SAD per block;
 * mv_i32: [nby*nbx][2] = (dy,dx) of the minimiser with the lowest raster index
 * (dy+R)*(2R+1)+(dx+R).  Reference reads outside the frame are clamped to the
 * edge.  (.) = Eq. 4, reference displaced as in Eq. 8. */
merit_status merit_sad_search(const merit_plan *plan, const void *cur_u8, const void *ref_u8,
                              void *sad_i32, void *mv_i32, void *hip_stream);

/* x_f16: [N,C,H,W], w_f16: [C,kh,kw], y_f16: [N,C,OH,OW], binary16.  Exact fp16 products,
 * fp32 accumulation in window scan order, one rounding. */
merit_status merit_conv2d_depthwise(const merit_plan *plan, const void *x_f16, const void *w_f16,
                                    void *y_f16, void *hip_stream);

/* x1_f16, x2_f16: [N,C,H,W] binary16; y_f16: [N,H,W,2R+1,2R+1] binary16 (the index order
 * (p1,p2,p3,p4) of Eq. 8).  Exact fp16 products, fp32 accumulation, one rounding. */
merit_status merit_correlation(const merit_plan *plan, const void *x1_f16, const void *x2_f16,
                               void *y_f16, void *hip_stream);

const char *merit_status_string(merit_status s);

#ifdef __cplusplus
}
#endif
#endif /* MERIT_H */
