// Shared host/device helpers of the gfx950 Chipmunk kernels.  Internal: the
// public interface is include/chipmunk.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/chipmunk.h"

namespace chipmunk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4v;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define CHIPMUNK_LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))
#define CHIPMUNK_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// two floats -> packed bf16 pair (round to nearest even), lo in bits 0..15
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    bf16x2 v;
    v[0] = (__bf16)lo;
    v[1] = (__bf16)hi;
    return __builtin_bit_cast(uint32_t, v);
}

// Asynchronous 16-byte load from global memory straight into LDS: lane l of the
// wave deposits its 16 bytes at lds_wave_base + 16*l (lds_wave_base is a
// wave-uniform LDS byte address).  The global address is base + byte_offset
// with a per-lane 32-bit offset, which makes this a gather.  Completion is
// counted by vmcnt; the caller waits (wait_all_memory) before the barrier that
// publishes the tile.  Issued as inline assembly so that the compiler does not
// serialise later LDS reads of OTHER buffers behind the outstanding transfer.
__device__ __forceinline__ void load_global_to_lds_16B(const void* base, uint32_t byte_offset,
                                                       uint32_t lds_wave_base) {
    // base and lds_wave_base are wave-uniform by contract; readfirstlane pins them to scalar registers
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    const uint64_t ub = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(b >> 32)) << 32) |
                        (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)b);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(__builtin_amdgcn_readfirstlane(lds_wave_base)), "v"(byte_offset), "s"(ub)
                 : "memory");
}

// Raw buffer resource (no stride, no swizzle) over `bytes` bytes at `base`, both wave-uniform.  Loads through it
// are range-checked by the hardware on (per-lane offset + immediate offset): an access that starts at or beyond
// `bytes` returns zero instead of touching memory.
typedef __attribute__((ext_vector_type(4))) int i32x4;
__device__ __forceinline__ i32x4 raw_buffer_words(const void* base, uint32_t bytes) {
    const uint64_t b = reinterpret_cast<uint64_t>(base);
    i32x4 r;
    r[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)b);
    r[1] = __builtin_amdgcn_readfirstlane((int)((uint32_t)(b >> 32) & 0xffffu));
    r[2] = __builtin_amdgcn_readfirstlane((int)bytes);
    r[3] = 0x00020000;
    return r;
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const void* base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// The same asynchronous 16-byte load to LDS through a buffer resource: the global address is the buffer's base +
// the lane's byte_offset (range-checked against the buffer's size, so no clamp of the offset is needed to stay
// inside the tensor).  No "memory" clobber: the transfer is asynchronous anyway (what orders it against the reads
// of the tile it fills are the caller's explicit wait and barrier, which the compiler does not move a volatile
// asm across), and without the clobber the compiler may keep scheduling LDS reads of OTHER buffers across it.
__device__ __forceinline__ void load_buffer_to_lds_16B(i32x4 buffer, uint32_t byte_offset, uint32_t lds_wave_base) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_wave_base), "v"(byte_offset), "s"(buffer)
                 );
}

// LDS byte address of a __shared__ object, made wave-uniform
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)CHIPMUNK_LDS_PTR(p));
}

// Transposing LDS read of 16-bit elements.  Within each block of 16 lanes,
// lane i supplies the address of 4 consecutive elements: row i/4, columns
// 4*(i%4)..+3 of a 4x16 block; lane j receives column j of that block, i.e.
// element t of its result is the block's (row t, column j).
__device__ __forceinline__ short4v lds_read_tr16(const void* lds_ptr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) short4v*)(lds_ptr));
}

// max / sum over the four 16-lane rows of a wave, result in every lane
__device__ __forceinline__ float rows4_max(float x) {
    uint32_t u = __float_as_uint(x);
    auto s = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = fmaxf(__uint_as_float(s[0]), __uint_as_float(s[1]));
    u = __float_as_uint(x);
    auto t = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__uint_as_float(t[0]), __uint_as_float(t[1]));
}
__device__ __forceinline__ float rows4_sum(float x) {
    uint32_t u = __float_as_uint(x);
    auto s = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    x = __uint_as_float(s[0]) + __uint_as_float(s[1]);
    u = __float_as_uint(x);
    auto t = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return __uint_as_float(t[0]) + __uint_as_float(t[1]);
}

__device__ __forceinline__ void wait_all_memory() { __builtin_amdgcn_s_waitcnt(0); }

// Waits until at most N of the wave's vector memory loads (the asynchronous LDS transfers among them) are still
// outstanding; they complete in the order they were issued.  (s_waitcnt: the count is split over bits 3:0 and
// 15:14; the export and LDS/scalar counters are left at their maxima.)
template <int N>
__device__ __forceinline__ void wait_vmem_at_most() {
    static_assert(N >= 0 && N < 64, "the counter has six bits");
    __builtin_amdgcn_s_waitcnt((N & 0xf) | ((N >> 4) << 14) | 0x0070 | 0x0f00);
}

// Workgroup barrier for data exchanged through LDS: waits for this wave's LDS accesses only, so that loads from
// global memory into registers stay in flight across it (__syncthreads() waits for those as well).
__device__ __forceinline__ void lds_accesses_then_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" : : : "memory");
}

// ---- host side ---------------------------------------------------------------

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Scalar arguments are classified on their bit patterns: these files are compiled without NaN semantics
// (-fno-honor-nans also covers the host half), so a comparison may be folded as if NaN did not exist.
inline uint32_t float_bits(float x) {
    uint32_t u;
    __builtin_memcpy(&u, &x, sizeof u);
    return u;
}
inline bool is_finite_scalar(float x) { return (float_bits(x) & 0x7f800000u) != 0x7f800000u; }
inline bool is_positive_finite_scalar(float x) {
    const uint32_t u = float_bits(x);
    return (u >> 31) == 0 && u != 0 && (u & 0x7f800000u) != 0x7f800000u;
}

inline int32_t launch_status() {
    return hipGetLastError() == hipSuccess ? CHIPMUNK_OK : CHIPMUNK_ERR_LAUNCH;
}

}  // namespace chipmunk
