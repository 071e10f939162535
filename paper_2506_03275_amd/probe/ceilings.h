/* Device-ceiling probes for gfx950: what the chip sustains for bare bf16 MFMA streams and for
 * streaming reads/copies.  Measurement aid for bench.py --ceilings; not part of the Chipmunk path
 * (nothing in libchipmunk_hip.so depends on it).  All pointers are device pointers owned by the
 * caller; every call enqueues one kernel on `stream` and returns 0, or -1 on a bad argument,
 * -6 on a launch error. */
#ifndef CHIPMUNK_CEILINGS_H
#define CHIPMUNK_CEILINGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Floating-point operations one launch of chipmunk_probe_mfma_bf16 performs (0 on a bad argument). */
double chipmunk_probe_mfma_flops(int blocks_per_cu, int iters);

/* Every wave runs `iters` rounds of 393216 flop of independent register-only bf16 MFMAs.
 *   shape: 16 -> 24 x v_mfma_f32_16x16x32_bf16 per round, 32 -> 12 x v_mfma_f32_32x32x16_bf16
 *   blocks_per_cu: 1 or 2 workgroups of 4 waves per compute unit (= waves per SIMD)
 *   sink: at least 2 * 256 * (number of compute units) floats, written once per thread */
int32_t chipmunk_probe_mfma_bf16(int shape, int blocks_per_cu, int iters, float* sink, void* stream);

/* Reads `bytes` (multiple of 16) once with 16-byte loads, eight in flight per lane. */
int32_t chipmunk_probe_read(const void* src, size_t bytes, float* sink, void* stream);

/* dst[0:bytes] = src[0:bytes] with 16-byte loads and stores (bytes multiple of 16, no overlap). */
int32_t chipmunk_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
