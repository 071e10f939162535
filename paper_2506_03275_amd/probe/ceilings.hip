// Device-ceiling probes for gfx950 (see ceilings.h).  Register-only MFMA streams and plain
// streaming kernels: they touch no memory beyond the buffers the caller passes.
#include <hip/hip_runtime.h>

#include "ceilings.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr double kFlopsPerRound = 24.0 * 16 * 16 * 32 * 2;  // = 12 * 32*32*16*2

__device__ __forceinline__ void probe_operands(bf16x8& a, bf16x8& b) {
    for (int t = 0; t < 8; t++) {
        a[t] = (__bf16)(((threadIdx.x * 7 + t * 3) % 13) * 0.01f - 0.06f);
        b[t] = (__bf16)(((threadIdx.x * 5 + t) % 11) * 0.02f - 0.1f);
    }
}

__global__ __launch_bounds__(256) void mfma16_kernel(float* sink, int iters) {
    bf16x8 a, b;
    probe_operands(a, b);
    f32x4 acc[24];
    for (int i = 0; i < 24; i++) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 24; i++) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 24; i++) s += acc[i][0] + acc[i][3];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void mfma32_kernel(float* sink, int iters) {
    bf16x8 a, b;
    probe_operands(a, b);
    f32x16 acc[12];
    for (int i = 0; i < 12; i++)
        for (int r = 0; r < 16; r++) acc[i][r] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int i = 0; i < 12; i++) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 12; i++) s += acc[i][0] + acc[i][7];
    sink[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void read_kernel(const float4* __restrict__ x, size_t n4, float* sink) {
    constexpr int U = 8;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    float acc = 0.f;
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n4; i += stride) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            size_t j = i + (size_t)u * 256;
            v[u] = x[j < n4 ? j : n4 - 1];
        }
#pragma unroll
        for (int u = 0; u < U; u++) acc += v[u].x + v[u].y + v[u].z + v[u].w;
    }
    if (acc == 12345.678f) sink[0] = acc;  // keeps the loads; never true for the buffers bench.py passes
}

__global__ __launch_bounds__(256) void copy_kernel(const float4* __restrict__ x, float4* __restrict__ y, size_t n4) {
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * 256 * U;
    for (size_t i = (size_t)blockIdx.x * 256 * U + threadIdx.x; i < n4; i += stride) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            size_t j = i + (size_t)u * 256;
            v[u] = x[j < n4 ? j : n4 - 1];
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            size_t j = i + (size_t)u * 256;
            if (j < n4) y[j] = v[u];
        }
    }
}

int compute_units() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return 0;
    return cus;
}

int32_t status() { return hipGetLastError() == hipSuccess ? 0 : -6; }

}  // namespace

extern "C" double chipmunk_probe_mfma_flops(int blocks_per_cu, int iters) {
    if ((blocks_per_cu != 1 && blocks_per_cu != 2) || iters < 1) return 0.0;
    return kFlopsPerRound * 4.0 * (double)compute_units() * blocks_per_cu * iters;
}

extern "C" int32_t chipmunk_probe_mfma_bf16(int shape, int blocks_per_cu, int iters, float* sink, void* stream) {
    if (!sink || iters < 1 || (blocks_per_cu != 1 && blocks_per_cu != 2)) return -1;
    if (shape != 16 && shape != 32) return -1;
    const int cus = compute_units();
    if (cus < 1) return -6;
    dim3 grid((unsigned)(cus * blocks_per_cu)), block(256);
    hipStream_t s = (hipStream_t)stream;
    if (shape == 16) hipLaunchKernelGGL(mfma16_kernel, grid, block, 0, s, sink, iters);
    else hipLaunchKernelGGL(mfma32_kernel, grid, block, 0, s, sink, iters);
    return status();
}

extern "C" int32_t chipmunk_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
    if (!src || !sink || bytes < 16 || (bytes & 15) || (reinterpret_cast<uintptr_t>(src) & 15)) return -1;
    hipLaunchKernelGGL(read_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const float4*)src, bytes / 16, sink);
    return status();
}

extern "C" int32_t chipmunk_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
    if (!src || !dst || bytes < 16 || (bytes & 15)) return -1;
    if ((reinterpret_cast<uintptr_t>(src) & 15) || (reinterpret_cast<uintptr_t>(dst) & 15)) return -1;
    hipLaunchKernelGGL(copy_kernel, dim3(4096), dim3(256), 0, (hipStream_t)stream, (const float4*)src, (float4*)dst,
                       bytes / 16);
    return status();
}
