// Max pooling of a binary16 tensor with a 3x3 window, stride 2, padding 1 (k = (n, c, py, px |
// ky, kx), c[n, c, 2 py + ky - 1, 2 px + kx - 1], -inf outside; the maximum as the product
// function of Section III-B): the second pass of a convolution + pooling plan whose layer is
// compute-bound, where pooling inside the convolution kernel costs more MFMA time (bands of
// pooled rows recompute the rows above them, tiles are whole rows) than one more trip of the
// convolution's result through the cache hierarchy.  HBM- / L2-bound: no LDS, no barrier.
//
// merit_maxpool_f16_k3s2p1_rows<V> (OW % V == 0, V = 8 or 4): a thread owns V input columns of two
// pooled rows: five input rows, each one V-half load plus the column to the left, the 3-maxima
// along the row at stride 2 on packed pairs, then down the rows; V/2 pooled pixels per row leave
// as one 8- or 4-byte store.  merit_maxpool_f16_k3s2p1 (any even OW): two pooled pixels per thread.
// The maxima are exact (values are only compared), so the result equals what the fused kernels write.
#include "merit_internal.h"

namespace merit {

namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t max_f16x2(uint32_t a, uint32_t b)
{
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(half2v, a), __builtin_bit_cast(half2v, b)));
}

}  // namespace

__global__ __launch_bounds__(256) void merit_maxpool_f16_k3s2p1(const uint16_t *__restrict__ c, uint16_t *__restrict__ y,
                                                                long long total, int OH, int OW, int PH, int PW,
                                                                int pairs)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    // idx = (plane * PH + py) * pairs + j; planes * PH stays below 2^31 (checked by the launcher)
    const uint32_t row = (uint32_t)(idx / pairs);
    const int j = (int)(idx - (long long)row * pairs);
    const uint32_t plane = row / (uint32_t)PH;
    const int py = (int)(row - plane * (uint32_t)PH);
    constexpr uint32_t NEG = 0xFC00FC00u;                   // two binary16 -inf
    const int x0 = 4 * j;                                   // first of the four columns read as dwords
    const bool has_left = x0 > 0, has_right = x0 + 2 < OW;  // column 4j-1 / columns 4j+2, 4j+3 exist (OW is even)
    uint32_t m_l = NEG, m_a = NEG, m_b = NEG;               // running maxima: column 4j-1 | 4j, 4j+1 | 4j+2, 4j+3
#pragma unroll
    for (int dr = -1; dr <= 1; ++dr) {
        const int r = 2 * py + dr;                          // r <= OH - 1 always (OH = 2 PH)
        if (r < 0) continue;
        const uint16_t *src = c + ((size_t)plane * OH + r) * OW + x0;
        const uint32_t a = *reinterpret_cast<const uint32_t *>(src);
        const uint32_t b = has_right ? *reinterpret_cast<const uint32_t *>(src + 2) : NEG;
        const uint32_t l = has_left ? (uint32_t)src[-1] | 0xFC000000u : NEG;
        m_a = max_f16x2(m_a, a);
        m_b = max_f16x2(m_b, b);
        m_l = max_f16x2(m_l, l);
    }
    // pooled pixel 2j: columns 4j-1, 4j, 4j+1; pooled pixel 2j+1: columns 4j+1, 4j+2, 4j+3
    const uint32_t a_hi = m_a >> 16;                        // column 4j+1
    const uint32_t first = max_f16x2(max_f16x2(m_l & 0xffffu, m_a & 0xffffu), a_hi) & 0xffffu;
    const uint32_t second = max_f16x2(max_f16x2(a_hi, m_b & 0xffffu), m_b >> 16) & 0xffffu;
    uint16_t *dst = y + ((size_t)plane * PH + py) * PW + 2 * j;
    dst[0] = (uint16_t)first;
    if (2 * j + 1 < PW) dst[1] = (uint16_t)second;
}

// { m_2j, m_2j+1 } for the V/2 pooled pixels of one input row: d[i] = columns (2i, 2i+1) of the
// thread's V columns, left = the column before them (low half)
template <int V>
__device__ __forceinline__ void row_max3(const uint32_t (&d)[V / 2], uint32_t left, uint32_t (&o)[V / 4])
{
#pragma unroll
    for (int j = 0; j < V / 4; ++j) {
        const uint32_t before = j == 0 ? left : (d[2 * j - 1] >> 16);                   // column 4j-1 in the low half
        const uint32_t ev = __builtin_amdgcn_perm(d[2 * j + 1], d[2 * j], 0x05040100u);  // columns 4j, 4j+2
        const uint32_t od = __builtin_amdgcn_perm(d[2 * j + 1], d[2 * j], 0x07060302u);  // columns 4j+1, 4j+3
        const uint32_t pv = (before & 0xffffu) | (d[2 * j] & 0xffff0000u);               // columns 4j-1, 4j+1
        o[j] = max_f16x2(max_f16x2(ev, od), pv);
    }
}

template <int V>
__global__ __launch_bounds__(256) void merit_maxpool_f16_k3s2p1_rows(const uint16_t *__restrict__ c, uint16_t *__restrict__ y,
                                                                     long long total, int OH, int OW, int PH, int PW)
{
    constexpr uint32_t NEG = 0xFC00FC00u;
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const int groups = OW / V, QH = (PH + 1) >> 1;          // column groups per row, pooled row pairs per plane
    const uint32_t rowq = (uint32_t)(idx / groups);         // plane * QH + q
    const int g = (int)(idx - (long long)rowq * groups);
    const uint32_t plane = rowq / (uint32_t)QH;
    const int q = (int)(rowq - plane * (uint32_t)QH);
    const uint16_t *base = c + (size_t)plane * OH * OW + V * g;
    uint32_t h[5][V / 4];
#pragma unroll
    for (int k = 0; k < 5; ++k) {
        const int r = 4 * q - 1 + k;
        uint32_t d[V / 2];
        uint32_t left = NEG;
        if (r >= 0 && r < OH) {
            const uint16_t *src = base + (size_t)r * OW;
            if constexpr (V == 8) {
                const uint4 v = *reinterpret_cast<const uint4 *>(src);
                d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
            } else {
                const uint2 v = *reinterpret_cast<const uint2 *>(src);
                d[0] = v.x; d[1] = v.y;
            }
            if (g > 0) left = src[-1];
            else left = 0xFC00u;
        } else {
#pragma unroll
            for (int i = 0; i < V / 2; ++i) d[i] = NEG;
        }
        row_max3<V>(d, left, h[k]);
    }
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int py = 2 * q + half;
        if (py >= PH) break;
        uint32_t o[V / 4];
#pragma unroll
        for (int j = 0; j < V / 4; ++j) o[j] = max_f16x2(max_f16x2(h[2 * half][j], h[2 * half + 1][j]), h[2 * half + 2][j]);
        uint16_t *dst = y + ((size_t)plane * PH + py) * PW + (V / 2) * g;
        if constexpr (V == 8) *reinterpret_cast<uint2 *>(dst) = make_uint2(o[0], o[1]);
        else *reinterpret_cast<uint32_t *>(dst) = o[0];
    }
}

// c: [planes][OH][OW] binary16 (OH, OW even), y: [planes][OH/2][OW/2]
hipError_t launch_maxpool_f16(const void *c, void *y, int64_t planes, int OH, int OW, hipStream_t s)
{
    const int PH = OH / 2, PW = OW / 2;
    const int pairs = (PW + 1) / 2;
    const int64_t rows = planes * PH;
    if (planes <= 0) return hipSuccess;
    if ((OH & 1) || (OW & 1) || rows >= (1ll << 31)) return hipErrorInvalidValue;
    if ((OW & 3) == 0) {
        const int V = (OW & 7) == 0 ? 8 : 4;
        const int64_t rowq = planes * ((PH + 1) / 2);
        const long long tot = (long long)rowq * (OW / V);
        const long long gr = (tot + 255) / 256;
        if (gr >= (1ll << 31)) return hipErrorInvalidValue;
        if (V == 8)
            hipLaunchKernelGGL(merit_maxpool_f16_k3s2p1_rows<8>, dim3((uint32_t)gr), dim3(256), 0, s,
                               static_cast<const uint16_t *>(c), static_cast<uint16_t *>(y), tot, OH, OW, PH, PW);
        else
            hipLaunchKernelGGL(merit_maxpool_f16_k3s2p1_rows<4>, dim3((uint32_t)gr), dim3(256), 0, s,
                               static_cast<const uint16_t *>(c), static_cast<uint16_t *>(y), tot, OH, OW, PH, PW);
        return hipGetLastError();
    }
    const long long total = (long long)rows * pairs;
    const long long grid = (total + 255) / 256;
    if (grid >= (1ll << 31)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(merit_maxpool_f16_k3s2p1, dim3((uint32_t)grid), dim3(256), 0, s,
                       static_cast<const uint16_t *>(c), static_cast<uint16_t *>(y), total, OH, OW, PH, PW, pairs);
    return hipGetLastError();
}

}  // namespace merit
