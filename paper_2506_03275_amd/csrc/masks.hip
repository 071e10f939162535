// Bit-packed column masks (App. B.4: the sparsity pattern of a layer is cached as one bit per (chunk, column)
// instead of one byte or one index) and their conversion to the index lists the delta kernels walk (Table 3:
// "mask to indices conversion", one fused kernel).  One workgroup per row; a row of C columns is ceil(C / 32)
// words, bit (j % 32) of word j / 32 set when column j is selected.
#include "common.h"

namespace chipmunk {

// inclusive prefix sum over the 64 lanes of a wave (DPP row shifts, then the lower rows' totals)
__device__ __forceinline__ uint32_t mask_wave_scan(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
    const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
    const int row = (threadIdx.x & 63) >> 4;
    return v + (row > 0 ? t0 : 0u) + (row > 1 ? t1 : 0u) + (row > 2 ? t2 : 0u);
}

// idx[r, 0:counts[r]] = the set bits of row r in ascending order; counts[r] = min(number of set bits, k_stride).
// Thread t owns the words [t * wpt, (t + 1) * wpt): one scan over the threads' bit counts gives every thread the
// output position of its first bit.
__global__ __launch_bounds__(256) void mask_to_indices_kernel(const uint32_t* __restrict__ mask, int64_t ld_words, int C,
                                                              int32_t* __restrict__ idx, int32_t* __restrict__ counts,
                                                              int k_stride) {
    __shared__ uint32_t s_wave[4];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t row = blockIdx.x;
    const uint32_t* m = mask + row * ld_words;
    const int words = (C + 31) >> 5;
    const int wpt = (words + 255) >> 8;                       // words per thread
    const int w0 = min(words, tid * wpt), w1 = min(words, w0 + wpt);
    const uint32_t tail = (C & 31) ? ((1u << (C & 31)) - 1u) : 0xffffffffu;   // bits of the last word that are columns
    uint32_t mine = 0;
    for (int i = w0; i < w1; i++) mine += __popc(m[i] & (i == words - 1 ? tail : 0xffffffffu));
    const uint32_t inc = mask_wave_scan(mine);
    if (lane == 63) s_wave[w] = inc;
    __syncthreads();
    const uint32_t t0 = s_wave[0], t1 = s_wave[1], t2 = s_wave[2], t3 = s_wave[3];
    uint32_t pos = inc - mine + (w > 0 ? t0 : 0u) + (w > 1 ? t1 : 0u) + (w > 2 ? t2 : 0u);
    if (tid == 0) counts[row] = (int32_t)min(t0 + t1 + t2 + t3, (uint32_t)k_stride);
    int32_t* out = idx + row * (int64_t)k_stride;
    for (int i = w0; i < w1; i++) {
        uint32_t bits = m[i] & (i == words - 1 ? tail : 0xffffffffu);
        while (bits) {
            if (pos < (uint32_t)k_stride) out[pos] = i * 32 + __ffs((int)bits) - 1;
            pos++;
            bits &= bits - 1;
        }
    }
}

// mask row r = the columns idx[r, 0:counts[r]] (entries outside [0, C) are ignored; a column listed twice sets
// its bit once).  The row is cleared and the bits are set in LDS, then written out whole.
__global__ __launch_bounds__(256) void indices_to_mask_kernel(const int32_t* __restrict__ idx,
                                                              const int32_t* __restrict__ counts, int C, int k_stride,
                                                              uint32_t* __restrict__ mask, int64_t ld_words) {
    extern __shared__ uint32_t s_bits[];
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const int words = (C + 31) >> 5;
    for (int i = tid; i < words; i += 256) s_bits[i] = 0u;
    __syncthreads();
    const int count = min(max(counts[row], 0), k_stride);
    const int32_t* in = idx + row * (int64_t)k_stride;
    for (int j = tid; j < count; j += 256) {
        const int col = in[j];
        if (col >= 0 && col < C) atomicOr(&s_bits[col >> 5], 1u << (col & 31));
    }
    __syncthreads();
    uint32_t* out = mask + row * ld_words;
    for (int i = tid; i < words; i += 256) out[i] = s_bits[i];
}

constexpr int kMaxMaskColumns = 1 << 20;   // 128 KB of LDS bits per row

}  // namespace chipmunk

using namespace chipmunk;

extern "C" int32_t chipmunk_mask_to_indices(const uint32_t* mask, int64_t ld_words, int R, int C, int32_t* idx,
                                            int32_t* counts, int k_stride, void* stream) {
    if (!mask || !idx || !counts) return CHIPMUNK_ERR_NULL;
    if (R < 1 || C < 1 || k_stride < 0 || ld_words < (C + 31) / 32) return CHIPMUNK_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(mask) & 3u) || (reinterpret_cast<uintptr_t>(idx) & 3u) ||
        (reinterpret_cast<uintptr_t>(counts) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    hipLaunchKernelGGL(mask_to_indices_kernel, dim3((unsigned)R), dim3(256), 0, (hipStream_t)stream, mask, ld_words, C, idx,
                       counts, k_stride);
    return launch_status();
}

extern "C" int32_t chipmunk_indices_to_mask(const int32_t* idx, const int32_t* counts, int R, int C, int k_stride,
                                            uint32_t* mask, int64_t ld_words, void* stream) {
    if (!mask || !idx || !counts) return CHIPMUNK_ERR_NULL;
    if (R < 1 || C < 1 || C > kMaxMaskColumns || k_stride < 0 || ld_words < (C + 31) / 32) return CHIPMUNK_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(mask) & 3u) || (reinterpret_cast<uintptr_t>(idx) & 3u) ||
        (reinterpret_cast<uintptr_t>(counts) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    const size_t lds = (size_t)((C + 31) / 32) * sizeof(uint32_t);
    if (hipFuncSetAttribute((const void*)indices_to_mask_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess)
        return CHIPMUNK_ERR_LAUNCH;
    hipLaunchKernelGGL(indices_to_mask_kernel, dim3((unsigned)R), dim3(256), lds, (hipStream_t)stream, idx, counts, C,
                       k_stride, mask, ld_words);
    return launch_status();
}
