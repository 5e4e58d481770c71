// Peak probes: a streaming copy and register-only instruction loops, for the measured-achievable
// peaks that the roofline fractions of the MERIT kernels are quoted beside.
#include "merit_internal.h"
#include "merit_probe.h"

namespace merit {

typedef float float4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));

__global__ __launch_bounds__(256) void merit_probe_copy_kernel(const float4v *__restrict__ src,
                                                              float4v *__restrict__ dst, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    for (size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x; i < n16; i += stride) {
        float4v v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + 256 * k < n16) v[k] = __builtin_nontemporal_load(src + i + 256 * k);
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (i + 256 * k < n16) __builtin_nontemporal_store(v[k], dst + i + 256 * k);
    }
}

template <int WHICH>
__global__ __launch_bounds__(256) void merit_probe_alu_kernel(int iters, uint32_t *__restrict__ sink)
{
    const uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x;
    uint32_t out = 0;
    if (WHICH == MERIT_PROBE_MFMA_F16) {
        floatx16 acc[8];
        half8 a, b;
#pragma unroll
        for (int j = 0; j < 8; ++j) { a[j] = (_Float16)(float)((seed >> j) & 3); b[j] = (_Float16)0.5f; }
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[c], 0, 0, 0);
        }
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s += acc[c][0] + acc[c][15];
        out = __builtin_bit_cast(uint32_t, s);
    } else if (WHICH == MERIT_PROBE_MFMA_F16_RANDOM) {
        // the same instruction stream on operands like a layer's: four operand pairs of hashed
        // binary16 values (random sign and mantissa, magnitudes 1/8 .. 1) taken in turn, so that
        // the multipliers see different bits every instruction
        floatx16 acc[8];
        half8 a[4], b[4];
        uint32_t hsh = seed | 1u;
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                hsh = hsh * 1664525u + 1013904223u;
                const uint16_t ba = (uint16_t)(((hsh >> 16) & 0x83ffu) | (uint16_t)((12 + ((hsh >> 28) & 3)) << 10));
                hsh = hsh * 1664525u + 1013904223u;
                const uint16_t bb = (uint16_t)(((hsh >> 16) & 0x83ffu) | (uint16_t)((12 + ((hsh >> 28) & 3)) << 10));
                a[k][j] = __builtin_bit_cast(_Float16, ba);
                b[k][j] = __builtin_bit_cast(_Float16, bb);
            }
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[c & 3], b[(c + (c >> 2)) & 3], acc[c], 0, 0, 0);
        }
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s += acc[c][0] + acc[c][15];
        out = __builtin_bit_cast(uint32_t, s);
    } else if (WHICH == MERIT_PROBE_FMA_F32) {
        float acc[8];
        const float m = 1.0f + (float)(seed & 7) * 1e-7f, d = (float)(seed & 3) * 1e-3f;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = (float)c;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = fmaf(acc[c], m, d);
        }
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s += acc[c];
        out = __builtin_bit_cast(uint32_t, s);
    } else if (WHICH == MERIT_PROBE_SAD_U8) {
        uint32_t acc[8];
        const uint32_t p = seed, q = seed ^ 0x5a5a5a5au;
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = c;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_sad_u8(p + c, q, acc[c]);
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) out += acc[c];
    } else {
        float acc[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[c] = -1.0f - (float)((seed + c) & 15) * 0.01f;
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] = __builtin_amdgcn_exp2f(acc[c]);     // stays in (0.4, 1)
        }
        float s = 0.0f;
#pragma unroll
        for (int c = 0; c < 8; ++c) s += acc[c];
        out = __builtin_bit_cast(uint32_t, s);
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = out;
}

}  // namespace merit

extern "C" {

merit_status merit_probe_copy(const void *src, void *dst, size_t bytes, void *stream)
{
    if (bytes == 0) return MERIT_OK;
    if (!src || !dst) return MERIT_ERR_NULL;
    if ((bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return MERIT_ERR_ALIGNMENT;
    const size_t n16 = bytes >> 4;
    size_t grid = (n16 + 1023) / 1024;
    if (grid > 256 * 32) grid = 256 * 32;
    hipLaunchKernelGGL(merit::merit_probe_copy_kernel, dim3((uint32_t)grid), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const merit::float4v *>(src),
                       static_cast<merit::float4v *>(dst), n16);
    return hipGetLastError() == hipSuccess ? MERIT_OK : MERIT_ERR_HIP;
}

merit_status merit_probe_alu(int which, int workgroups, int iters, void *sink, void *stream)
{
    if (which < 0 || which > 4 || workgroups < 0 || iters < 0 || workgroups > (1 << 20)) return MERIT_ERR_INVALID_ARG;
    if (workgroups == 0) return MERIT_OK;
    if (!sink) return MERIT_ERR_NULL;
    if ((uintptr_t)sink & 3) return MERIT_ERR_ALIGNMENT;
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint32_t *out = static_cast<uint32_t *>(sink);
    const dim3 g((uint32_t)workgroups), b(256);
    switch (which) {
    case MERIT_PROBE_MFMA_F16:
        hipLaunchKernelGGL(merit::merit_probe_alu_kernel<MERIT_PROBE_MFMA_F16>, g, b, 0, s, iters, out); break;
    case MERIT_PROBE_FMA_F32:
        hipLaunchKernelGGL(merit::merit_probe_alu_kernel<MERIT_PROBE_FMA_F32>, g, b, 0, s, iters, out); break;
    case MERIT_PROBE_SAD_U8:
        hipLaunchKernelGGL(merit::merit_probe_alu_kernel<MERIT_PROBE_SAD_U8>, g, b, 0, s, iters, out); break;
    case MERIT_PROBE_MFMA_F16_RANDOM:
        hipLaunchKernelGGL(merit::merit_probe_alu_kernel<MERIT_PROBE_MFMA_F16_RANDOM>, g, b, 0, s, iters, out); break;
    default:
        hipLaunchKernelGGL(merit::merit_probe_alu_kernel<MERIT_PROBE_EXP2_F32>, g, b, 0, s, iters, out); break;
    }
    return hipGetLastError() == hipSuccess ? MERIT_OK : MERIT_ERR_HIP;
}

}  // extern "C"
