// The ranged inner product for any descriptor (Section III, Eq. 1; Section III-C, Eq. 5), as the
// definition reads: one thread per row p of M(A) and M(B), a loop over the accumulation range a,
//     x_i = sum_j delta(i, d_j) (k_j s_j + o_j),   k = (p, a),
// for both operands, the padding rule where a coordinate leaves its tensor, and the product
// function of the plan's operation:
//     dot product (binary16 operands, fp32 sum, optional clip, one rounding to binary16),
//     maximum, or mean over the elements that are there (fp32).
// Nothing is staged and nothing is tiled: this is the kernel a descriptor gets that none of the
// specialised kernels recognises (a flipped or strided window, windows over more than two axes,
// a matrix product written as a transform, a dilated pooling window, a correlation layer whose
// width the MFMA kernel does not take).  Consecutive threads take consecutive rows p, the last
// parallel index fastest, so whatever that index moves along is read coalesced.
#include "merit_internal.h"

namespace merit {

namespace {

__device__ __forceinline__ float half_to_float(uint16_t h)
{
    return (float)__builtin_bit_cast(_Float16, h);
}

struct Coord {
    int x[MERIT_MAX_DIMS];
};

// value of operand `o` at coordinate c, with the padding rule; `in` says whether c is inside
template <typename T>
__device__ __forceinline__ T fetch(const GenericOperand &o, const T *base, const Coord &c, int pad, bool &in)
{
    in = true;
    long long off = 0;
#pragma unroll
    for (int i = 0; i < MERIT_MAX_DIMS; ++i) {
        if (i >= o.ndim) break;
        int xi = c.x[i];
        if (xi < 0 || xi >= o.shape[i]) {
            in = false;
            xi = min(max(xi, 0), o.shape[i] - 1);          // the nearest element (used by the clamp rule only)
        }
        off += (long long)xi * o.pitch[i];
    }
    if (!in && pad != MERIT_PAD_CLAMP) return T(0);
    return base[off];
}

}  // namespace

// MODE 0: dot product, 1: maximum, 2: mean
template <int MODE>
__global__ __launch_bounds__(256) void merit_generic(GenericParams p, const void *__restrict__ a_,
                                                    const void *__restrict__ b_, void *__restrict__ y_)
{
    const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
    if (row >= p.rows) return;
    // row -> parallel indices, last fastest; their share of every coordinate
    Coord ca, cb;
#pragma unroll
    for (int i = 0; i < MERIT_MAX_DIMS; ++i) ca.x[i] = cb.x[i] = 0;
    {
        long long r = row;
        for (int j = p.n_par - 1; j >= 0; --j) {
            const long long q = r / p.range[j];
            const int k = (int)(r - q * p.range[j]);
            r = q;
            if (p.a.axis[j] >= 0) ca.x[p.a.axis[j]] += k * p.a.stride[j] + p.a.offset[j];
            if (MODE == 0 && p.b.axis[j] >= 0) cb.x[p.b.axis[j]] += k * p.b.stride[j] + p.b.offset[j];
        }
        // the offsets of the accumulation indices do not depend on their value either
        for (int j = p.n_par; j < p.n_par + p.n_acc; ++j) {
            if (p.a.axis[j] >= 0) ca.x[p.a.axis[j]] += p.a.offset[j];
            if (MODE == 0 && p.b.axis[j] >= 0) cb.x[p.b.axis[j]] += p.b.offset[j];
        }
    }
    // the accumulation range, last index fastest, as an odometer: a step adds the stride of the
    // index that moved and takes back the full travel of those that wrapped
    int k[MERIT_MAX_INDEX];
    for (int j = 0; j < p.n_acc; ++j) k[j] = 0;
    float sum = 0.0f, best = -__builtin_inff();
    long long count = 0;
    for (long long t = 0; t < p.acc; ++t) {
        bool ina, inb = true;
        if (MODE == 0) {
            const float va = half_to_float(fetch<uint16_t>(p.a, static_cast<const uint16_t *>(a_), ca, p.pad, ina));
            const float vb = half_to_float(fetch<uint16_t>(p.b, static_cast<const uint16_t *>(b_), cb, p.pad, inb));
            sum = __builtin_fmaf(va, vb, sum);
        } else {
            const float va = fetch<float>(p.a, static_cast<const float *>(a_), ca, p.pad, ina);
            const bool there = ina || p.pad == MERIT_PAD_CLAMP;
            if (MODE == 1) {
                if (there) best = fmaxf(best, va);
                else if (p.pad == MERIT_PAD_ZERO) best = fmaxf(best, 0.0f);
            } else {
                if (there || p.pad == MERIT_PAD_ZERO) { sum += va; ++count; }
            }
        }
        for (int j = p.n_acc - 1; j >= 0; --j) {
            const int jj = p.n_par + j;
            const int aa = p.a.axis[jj], ab = p.b.axis[jj];
            if (++k[j] < p.range[jj]) {
                if (aa >= 0) ca.x[aa] += p.a.stride[jj];
                if (MODE == 0 && ab >= 0) cb.x[ab] += p.b.stride[jj];
                break;
            }
            k[j] = 0;
            if (aa >= 0) ca.x[aa] -= (p.range[jj] - 1) * p.a.stride[jj];
            if (MODE == 0 && ab >= 0) cb.x[ab] -= (p.range[jj] - 1) * p.b.stride[jj];
        }
    }
    if (MODE == 0) {
        if (p.relu) sum = fmaxf(sum, 0.0f);
        static_cast<uint16_t *>(y_)[row] = __builtin_bit_cast(uint16_t, (_Float16)sum);
    } else if (MODE == 1) {
        static_cast<float *>(y_)[row] = best;
    } else {
        static_cast<float *>(y_)[row] = count > 0 ? sum / (float)count : 0.0f;
    }
}

hipError_t launch_generic(const GenericParams &p, const void *a, const void *b, void *y, hipStream_t s)
{
    if (p.rows == 0) return hipSuccess;
    const uint32_t grid = (uint32_t)((p.rows + 255) / 256);
    if (p.mode == 0) hipLaunchKernelGGL(merit_generic<0>, dim3(grid), dim3(256), 0, s, p, a, b, y);
    else if (p.mode == 1) hipLaunchKernelGGL(merit_generic<1>, dim3(grid), dim3(256), 0, s, p, a, b, y);
    else hipLaunchKernelGGL(merit_generic<2>, dim3(grid), dim3(256), 0, s, p, a, b, y);
    return hipGetLastError();
}

const char *generic_kernel_name(const GenericParams &p)
{
    return p.mode == 0 ? "merit_generic<dot>" : (p.mode == 1 ? "merit_generic<max>" : "merit_generic<mean>");
}

}  // namespace merit
