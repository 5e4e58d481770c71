/* Peak probes: what the chip sustains on the three resources the MERIT kernels are priced
 * against (memory stream, matrix cores, vector ALU), measured with kernels that do nothing
 * else.  For callers that report a roofline fraction and want the measured-achievable peak
 * beside the data-sheet one; no part of the MERIT path calls them.
 *
 * All pointers are device pointers owned by the caller; every call enqueues one kernel on
 * `hip_stream` (NULL = default stream) and returns; merit_status as in merit.h. */
#ifndef MERIT_PROBE_H
#define MERIT_PROBE_H

#include "merit.h"

#ifdef __cplusplus
extern "C" {
#endif

/* dst[0 .. bytes) = src[0 .. bytes), 16 bytes per lane and step, streaming loads and stores.
 * bytes must be a multiple of 16, both pointers 16-byte aligned.  Traffic: bytes read +
 * bytes written. */
merit_status merit_probe_copy(const void *src, void *dst, size_t bytes, void *hip_stream);

/* which: */
enum {
    MERIT_PROBE_MFMA_F16 = 0, /* v_mfma_f32_32x32x16_f16: 32768 flop per wavefront instruction */
    MERIT_PROBE_FMA_F32 = 1,  /* v_fma_f32 (not packed): 1 lane-op per lane                    */
    MERIT_PROBE_SAD_U8 = 2,   /* v_sad_u8: 1 lane-op (4 pixel differences) per lane            */
    MERIT_PROBE_EXP2_F32 = 3, /* v_exp_f32: 1 lane-op per lane                                 */
    MERIT_PROBE_MFMA_F16_RANDOM = 4 /* the MFMA loop on random binary16 operands (sign, mantissa and a few
                                 * exponents hashed per lane, four operand pairs in turn): what the matrix
                                 * cores sustain on data like a layer's, where the clock follows the power */
};

/* Runs `workgroups` workgroups of 256 threads; every wavefront issues iters x 8 instructions
 * of the chosen kind on eight independent register chains and finally writes one dword per
 * lane to sink (workgroups * 256 dwords), so that nothing is optimised away.  Instructions
 * issued in all: workgroups * 4 wavefronts * iters * 8. */
merit_status merit_probe_alu(int which, int workgroups, int iters, void *sink, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
