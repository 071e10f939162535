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

/* Every wave runs `iters` rounds of [393216 flop of independent bf16 MFMAs | valu_ops dependent-free
 * fp32 FMAs], the two groups kept apart as they are in a softmax-between-GEMMs loop.
 *   shape: 16 -> 24 x v_mfma_f32_16x16x32_bf16 per round, 32 -> 12 x v_mfma_f32_32x32x16_bf16
 *   blocks_per_cu: 1 or 2 workgroups of 4 waves per compute unit (= waves per SIMD)
 *   valu_ops: 0, 64 or 128
 *   sink: at least 2 * 256 * (number of compute units) floats, written once per thread */
int32_t chipmunk_probe_mfma_bf16(int shape, int blocks_per_cu, int valu_ops, int iters, float* sink, void* stream);

/* The stream of chipmunk_probe_mfma_bf16(16, blocks_per_cu, ~64, ...) with its two phases cut finer: every round is
 * 24 / mfmas_per_phase times [mfmas_per_phase x v_mfma_f32_16x16x32_bf16 | 60 * mfmas_per_phase / 24 fp32 FMAs]
 * (the same work per round whatever the cut).  mfmas_per_phase: 24, 12, 8, 4 or 2.  Flop of one launch:
 * chipmunk_probe_mfma_flops(blocks_per_cu, iters). */
int32_t chipmunk_probe_mfma_phases(int mfmas_per_phase, int blocks_per_cu, int iters, float* sink, void* stream);

/* The softmax-between-GEMMs instruction stream at its finest grain: every wave runs `iters` rounds of 24 slots, a
 * slot being 32768 flop of MFMA (one 32x32x16 or two 16x16x32, shape = 32 or 16).  head_dim = 64: every slot is
 * followed by the vector work of one pair of probabilities (2 multiply-subtracts, 2 exponentials, 1 bf16 pack), all
 * pinned in that order; head_dim = 128: every second slot (a score costs 4 * head_dim flop, so these are the
 * softmax's vector instructions per flop at that head dimension); head_dim = 0: MFMAs alone.
 * chipmunk_probe_mfma_slots_flops gives the flop of one launch. */
double chipmunk_probe_mfma_slots_flops(int blocks_per_cu, int iters);
int32_t chipmunk_probe_mfma_slots(int shape, int blocks_per_cu, int head_dim, int iters, float* sink,
                                  void* stream);

/* The tile-loading pattern of the GEMM kernels without arithmetic: 8 workgroups per compute unit in all, two
 * resident at a time, each running `steps` double-buffered steps of 40 KB of asynchronous 16-byte transfers to LDS
 * (320 pieces of 128 bytes, one per row of 6144 bytes; rows hashed over the first `rows` rows of src, which must
 * hold rows * 6144 bytes).  A small `rows` keeps the source in L2, a large one sends every piece beyond it.
 * chipmunk_probe_lds_fill_bytes gives the bytes one launch moves.  sink: 8 * 256 * (compute units) floats. */
double chipmunk_probe_lds_fill_bytes(int steps);
int32_t chipmunk_probe_lds_fill(const void* src, size_t src_bytes, uint32_t rows, int steps, float* sink, void* stream);

/* Reads `bytes` (multiple of 16) once with 16-byte loads, eight in flight per lane. */
int32_t chipmunk_probe_read(const void* src, size_t bytes, float* sink, void* stream);

/* dst[0:bytes] = src[0:bytes] with 16-byte loads and stores (bytes multiple of 16, no overlap). */
int32_t chipmunk_probe_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
