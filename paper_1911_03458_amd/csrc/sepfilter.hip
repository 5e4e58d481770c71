// Separable filter for gfx950: two 1-D ranged inner products in a row (dot product, Section
// III-B Eq. 3), the window centred as in the bilateral-filter call of Section VI-A (offset -k/2):
//     t[n,p1,p2] = sum_{a2<k} kx[a2] * x[n, p1, p2 + a2 - k/2]
//     y[n,p1,p2] = sum_{a1<k} ky[a1] * t[n, p1 + a1 - k/2, p2]
// with coordinates clamped to the image.  Both passes run in one launch and the intermediate
// t never leaves LDS (it overwrites the staged input there): 8 algorithmic bytes per pixel (one fp32 read, one fp32 written).
//
// A workgroup owns TH x 64 output pixels of one image.  The covering sub-tensor (Section IV-A,
// Eq. 9: (TH + k - 1) x (64 + k - 1)) is staged in LDS with the clamping resolved there.  A
// row-pass thread keeps 8 adjacent outputs of one staged row in registers and reads the
// 8 + k - 1 inputs they need as 16-byte runs; a column-pass thread keeps a 4 x 4 patch and
// reads k + 3 runs of four columns: 8k and 16k multiply-adds for that many 16-byte reads.
// In the row pass neighbouring lanes take neighbouring rows; the row pitches are 4 mod 8
// floats, which spreads the 16-byte accesses of 16 lanes over all banks (the padding layout
// of Section IV-B).
//
// The staged columns start at x0 - c4, c4 = k/2 rounded up to 4, so that (for W % 4 == 0) every
// group of four staged columns is one aligned 16-byte run of the image, entirely inside it or
// entirely outside (then it is four copies of the edge pixel): the staging is 16-byte loads
// without a branch, and the row pass reads its window c4 - k/2 columns further right.
#include "merit_internal.h"

namespace merit {

typedef float float4v __attribute__((ext_vector_type(4)));

// K = window length (compile time: every tap index is an immediate, the sliding windows live
// in renamed registers and no zero tap is multiplied)
template <int K>
__global__ __launch_bounds__(256, (K > 16 ? 3 : 1)) void merit_sepfilter_tile(SepParams p, const float *__restrict__ x,
                                                           const float *__restrict__ kx,
                                                           const float *__restrict__ ky, float *__restrict__ y)
{
    constexpr int TW = 64;
    constexpr int C = K / 2, C4 = (C + 3) / 4 * 4, D = C4 - C;    // staged column 0 = image column x0 - C4
    constexpr int NWR = (D + 8 + K - 1 + 3) / 4;                  // 16-byte groups a row-pass unit reads
    constexpr int K4 = (K + 3) / 4;
    constexpr int PR = 4;                                         // rows of a column-pass patch
    extern __shared__ __align__(16) float smem[];
    const int RH = p.TH + K - 1;                          // staged rows
    float *in = smem;                                     // [RH][PI]; later the row-pass result
    float *wxl = in + RH * p.PI;                          // [4*K4]
    float *wyl = wxl + 4 * K4;                            // [4*K4]

    const int tid = threadIdx.x;
    const int ntiles = p.N * p.tiles_y * p.tiles_x;
    struct Tile {
        int n, x0, y0;
    };
    auto tile_at = [&](int t) {
        const uint32_t q0 = fdiv((uint32_t)t, p.div_tiles_x);
        Tile T;
        T.n = (int)fdiv(q0, p.div_tiles_y);
        T.x0 = (t - (int)q0 * p.tiles_x) * TW;
        T.y0 = ((int)q0 - T.n * p.tiles_y) * p.TH;
        return T;
    };

    // The taps live in LDS and are read into vector registers at the start of each pass:
    // measured on gfx950, a multiply-add stream whose tap sits in a scalar register issues
    // one wavefront instruction per 4.2-4.6 clocks, with all operands in vector registers
    // one per 2.4-3.0 clocks (two or more wavefronts per SIMD).
    if (tid < 4 * K4) {
        wxl[tid] = tid < K ? kx[min(tid, K - 1)] : 0.0f;
        wyl[tid] = tid < K ? ky[min(tid, K - 1)] : 0.0f;
    }
    // Staging: every element is a real (clamped) pixel.  A thread owns one 4-column group of
    // the staged rows r = tid / LPR + (256 / LPR) j; SB rows per batch, every load of a batch
    // issued before the first LDS write (one memory round trip per batch).
    constexpr int SB = K <= 16 ? 8 : 12;                  // 8 rows per step: 64 or 96 staged rows at most
    const int P4 = p.PI >> 2, W4 = p.W >> 2;              // P4 <= 32 for every K <= 32
    const bool vec = (p.W & 3) == 0;
    constexpr int lg = 5;                                 // lanes per staged row
    const int cg = tid & ((1 << lg) - 1);
    const bool live = cg < P4;
    constexpr int rstep = 256 >> lg;
    // One batch covers a tile, so a workgroup requests its next tile before it computes the
    // current one: loads, arithmetic and stores of the workgroups of a compute unit overlap
    // instead of all running in the same phase.
    const bool pf = vec;
    float4v pre[SB];
    auto issue = [&](const Tile &T, int r0) {
        const int g4 = ((T.x0 - C4) >> 2) + cg;           // image 4-column group (may be outside)
        // uniform image base + 32-bit element offsets (the plan keeps H*W below 2^31)
        const float *img = x + (size_t)T.n * p.H * p.W;
        const uint32_t col = 4u * (uint32_t)min(max(g4, 0), W4 - 1);
#pragma unroll
        for (int b = 0; b < SB; ++b) {
            const int gy = min(max(T.y0 - C + r0 + rstep * b, 0), p.H - 1);
            pre[b] = *reinterpret_cast<const float4v *>(img + (col + (uint32_t)gy * (uint32_t)p.W));
        }
    };
    auto commit = [&](const Tile &T, int r0) {
        const int g4 = ((T.x0 - C4) >> 2) + cg;
        const bool inside = g4 >= 0 && g4 < W4;           // else: four copies of the edge pixel
        const bool left = g4 < 0;
#pragma unroll
        for (int b = 0; b < SB; ++b) {
            const int r = r0 + rstep * b;
            const float edge = left ? pre[b].x : pre[b].w;
            float4v o;
            o.x = inside ? pre[b].x : edge; o.y = inside ? pre[b].y : edge;
            o.z = inside ? pre[b].z : edge; o.w = inside ? pre[b].w : edge;
            if (live && r < RH) reinterpret_cast<float4v *>(in)[r * P4 + cg] = o;
        }
    };

    // Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  Every XCD sweeps its
    // own contiguous eighth of the raster-ordered tile list (a band of tile rows), its workgroups
    // side by side: horizontally adjacent tiles, which share the cache lines of their halo columns,
    // and vertically adjacent ones, which share k - 1 halo rows, meet in one L2 at about the same
    // time.  (With runs of four tiles per XCD in raster order over the whole chip the vertical
    // neighbours sat on other XCDs: 1.72 times the image was fetched at k = 30.)
    const int nwg = (int)gridDim.x;
    int t = (int)blockIdx.x, tstep = nwg, tend = ntiles;
    if (nwg % 8 == 0) {
        const int xcd = t & 7, slot = t >> 3;
        t = (int)(((long long)xcd * ntiles) >> 3) + slot;         // slot < nwg / 8 <= the band's length
        tend = (int)(((long long)(xcd + 1) * ntiles) >> 3);
        tstep = nwg >> 3;
    }
    if (pf) issue(tile_at(t), tid >> lg);                 // t < tend: the grid never exceeds the tile list
    for (; t < tend; t += tstep) {
        const Tile T = tile_at(t);
        const int x0 = T.x0, y0 = T.y0;
        if (pf) {
            commit(T, tid >> lg);
        } else {
            const float *img = x + (size_t)T.n * p.H * p.W;
            const int total = RH * p.PI;
            for (int e = tid; e < total; e += 256) {
                const int r = e / p.PI;
                const int cc = e - r * p.PI;
                const int gy = min(max(y0 - C + r, 0), p.H - 1);
                const int gx = min(max(x0 - C4 + cc, 0), p.W - 1);
                in[e] = img[(size_t)gy * p.W + gx];
            }
        }
        __syncthreads();
        // short windows: the next tile's loads fly during both passes; long windows need the
        // registers for the row pass and request it before the column pass
        if (K <= 16 && pf && t + tstep < tend) issue(tile_at(t + tstep), tid >> lg);

        // row pass: unit = (8-column group, staged row), rows fastest; output column j of the
        // unit = sum_a kx[a] * staged column (8 cg + j + D + a).  The results replace the staged
        // input in place (columns 0..63 of each row): every unit is computed into registers
        // first, and a barrier separates the last read from the first write.
        constexpr int RU = K <= 16 ? 2 : 3;               // units per thread: 8 * RH <= 256 * RU
        float acc[RU][8];
        float wx[4 * K4];
#pragma unroll
        for (int g = 0; g < K4; ++g) {
            const float4v w = *reinterpret_cast<const float4v *>(wxl + 4 * g);
            wx[4 * g] = w.x; wx[4 * g + 1] = w.y; wx[4 * g + 2] = w.z; wx[4 * g + 3] = w.w;
        }
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            const int u = min(tid + 256 * k, (TW / 8) * RH - 1);
            const int cgr = (int)fdiv((uint32_t)u, p.div_rh);
            const int r = u - cgr * RH;
            const float *src = in + r * p.PI + 8 * cgr;
            float win[4 * NWR];
#pragma unroll
            for (int g = 0; g < NWR; ++g) {
                const float4v h = *reinterpret_cast<const float4v *>(src + 4 * g);
                win[4 * g] = h.x; win[4 * g + 1] = h.y; win[4 * g + 2] = h.z; win[4 * g + 3] = h.w;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k][j] = 0.0f;
#pragma unroll
            for (int a = 0; a < K; ++a)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[k][j] = fmaf(wx[a], win[j + D + a], acc[k][j]);
            // long windows: one unit's window at a time in registers.  The empty statement
            // consumes the sums and clobbers memory, so these multiply-adds stay above it and
            // the next unit's reads below it.
            if constexpr (K > 16)
                asm volatile("" : "+v"(acc[k][0]), "+v"(acc[k][1]), "+v"(acc[k][2]), "+v"(acc[k][3]),
                                  "+v"(acc[k][4]), "+v"(acc[k][5]), "+v"(acc[k][6]), "+v"(acc[k][7]) : : "memory");
        }
        __syncthreads();
        float *mid = in;                                  // [RH][PI], columns 0..63
#pragma unroll
        for (int k = 0; k < RU; ++k) {
            const int u = tid + 256 * k;
            if (u < (TW / 8) * RH) {
                const int cgr = (int)fdiv((uint32_t)u, p.div_rh);
                const int r = u - cgr * RH;
                float *dst = mid + r * p.PI + 8 * cgr;
                float4v o0, o1;
                o0.x = acc[k][0]; o0.y = acc[k][1]; o0.z = acc[k][2]; o0.w = acc[k][3];
                o1.x = acc[k][4]; o1.y = acc[k][5]; o1.z = acc[k][6]; o1.w = acc[k][7];
                *reinterpret_cast<float4v *>(dst) = o0;
                *reinterpret_cast<float4v *>(dst + 4) = o1;
            }
        }
        __syncthreads();
        if (K > 16 && pf && t + tstep < tend) issue(tile_at(t + tstep), tid >> lg);

        // column pass: unit = PR rows x 4 columns, column groups fastest: 16-byte LDS reads and
        // 16-byte stores.  Row q of the K + PR - 1 rows a unit reads feeds output row i with tap
        // q - i.
        float *out = y + (size_t)T.n * p.H * p.W;
        float wy[4 * K4];
#pragma unroll
        for (int g = 0; g < K4; ++g) {
            const float4v w = *reinterpret_cast<const float4v *>(wyl + 4 * g);
            wy[4 * g] = w.x; wy[4 * g + 1] = w.y; wy[4 * g + 2] = w.z; wy[4 * g + 3] = w.w;
        }
        for (int u = tid; u < (p.TH / PR) * (TW / 4); u += 256) {
            const int rg = u >> 4, c4 = u & 15;
            const float *src = mid + (PR * rg) * p.PI + 4 * c4;
            float4v o[PR];
#pragma unroll
            for (int i = 0; i < PR; ++i) o[i] = (float4v){0.0f, 0.0f, 0.0f, 0.0f};
            // QC rows at a time: their reads, then their multiply-adds (for long windows the
            // scheduler must not pull all K + 3 reads to the front: 4 registers each)
            constexpr int QC = K > 16 ? 4 : 8;
#pragma unroll
            for (int q0 = 0; q0 < K + PR - 1; q0 += QC) {
                float4v v[QC];
#pragma unroll
                for (int e = 0; e < QC; ++e)
                    if (q0 + e < K + PR - 1) v[e] = *reinterpret_cast<const float4v *>(src + (q0 + e) * p.PI);
#pragma unroll
                for (int e = 0; e < QC; ++e) {
                    const int q = q0 + e;
#pragma unroll
                    for (int i = 0; i < PR; ++i)
                        if (q < K + PR - 1 && q - i >= 0 && q - i < K) {
                            o[i].x = fmaf(wy[q - i], v[e].x, o[i].x);
                            o[i].y = fmaf(wy[q - i], v[e].y, o[i].y);
                            o[i].z = fmaf(wy[q - i], v[e].z, o[i].z);
                            o[i].w = fmaf(wy[q - i], v[e].w, o[i].w);
                        }
                }
                if constexpr (K > 16)
                    asm volatile("" : "+v"(o[0]), "+v"(o[1]), "+v"(o[2]), "+v"(o[3]) : : "memory");
            }
            const int gx = x0 + 4 * c4;
#pragma unroll
            for (int i = 0; i < PR; ++i) {
                const int gy = y0 + PR * rg + i;
                if (gy >= p.H) continue;
                float *dst = out + (size_t)gy * p.W + gx;
                if (vec) {
                    if (gx < p.W) *reinterpret_cast<float4v *>(dst) = o[i];
                } else {
                    if (gx < p.W) dst[0] = o[i].x;
                    if (gx + 1 < p.W) dst[1] = o[i].y;
                    if (gx + 2 < p.W) dst[2] = o[i].z;
                    if (gx + 3 < p.W) dst[3] = o[i].w;
                }
            }
        }
        __syncthreads();                                  // the staged tile is free again
    }
}

template <int K>
static hipError_t launch_sep(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                             hipStream_t s, int64_t ntiles, int cus)
{
    static std::atomic<int> raised{0};
    if (hipError_t e = raise_lds_limit_once(reinterpret_cast<const void *>(merit_sepfilter_tile<K>), raised);
        e != hipSuccess)
        return e;
    // Persistent workgroups.  The plan's count per CU is what LDS allows.  Long windows need so
    // many registers that fewer are resident, and a workgroup beyond the resident ones would
    // start only when another has finished all of its tiles: there the grid is exactly the
    // resident count (k = 30 at 4x1080x1920: 768 instead of 1024 workgroups, 30.2 -> 28.1 us).
    // Short windows keep the plan's count: one tile per workgroup, dealt out as workgroups
    // retire, measured faster than two rounds over the resident ones (k = 3: 17.2 against 17.9 us).
    int per_cu = p.wg_per_cu;
    if (K > 16) {
        // the last query and its answer in one atomic word (plans of one shape repeat); two
        // threads with different shapes at worst repeat the query, neither reads the other's answer
        static std::atomic<uint64_t> last{0};
        const uint64_t seen = last.load(std::memory_order_relaxed);
        int answer = (int)(seen & 0xffffffffu);
        if ((seen >> 32) != (uint64_t)(uint32_t)p.lds_bytes || answer <= 0) {
            int r = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&r, merit_sepfilter_tile<K>, 256,
                                                             (size_t)p.lds_bytes) != hipSuccess || r <= 0)
                r = 1;
            answer = r;
            last.store(((uint64_t)(uint32_t)p.lds_bytes << 32) | (uint32_t)r, std::memory_order_relaxed);
        }
        if (answer < per_cu) per_cu = answer;
    }
    const int64_t slots = (int64_t)cus * per_cu;
    const uint32_t grid = (uint32_t)(ntiles < slots ? ntiles : slots);
    hipLaunchKernelGGL(merit_sepfilter_tile<K>, dim3(grid), dim3(256), (size_t)p.lds_bytes, s, p, x, kx, ky, y);
    return hipGetLastError();
}

hipError_t launch_sepfilter(const SepParams &p, const float *x, const float *kx, const float *ky, float *y,
                            hipStream_t s)
{
    const int64_t ntiles = (int64_t)p.N * p.tiles_y * p.tiles_x;
    if (ntiles == 0) return hipSuccess;
    // persistent workgroups, p.wg_per_cu per compute unit (256 on MI355X), at most one per tile
    const int cus = device_cu_count();
    switch (p.k) {
#define MERIT_SEP_CASE(Kv) case Kv: return launch_sep<Kv>(p, x, kx, ky, y, s, ntiles, cus)
#define MERIT_SEP_CASE8(B)                                                                           \
    MERIT_SEP_CASE(B + 1); MERIT_SEP_CASE(B + 2); MERIT_SEP_CASE(B + 3); MERIT_SEP_CASE(B + 4);      \
    MERIT_SEP_CASE(B + 5); MERIT_SEP_CASE(B + 6); MERIT_SEP_CASE(B + 7); MERIT_SEP_CASE(B + 8)
        MERIT_SEP_CASE8(0); MERIT_SEP_CASE8(8); MERIT_SEP_CASE8(16); MERIT_SEP_CASE8(24);
#undef MERIT_SEP_CASE8
#undef MERIT_SEP_CASE
    default: return hipErrorInvalidValue;
    }
}

}  // namespace merit
