// Exact per-row top-k column selection (Sec. 3.3.1 idx = TopK_k(D); Alg. 7
// idx = TopK(|T - T_m|)) for gfx950.
//
// One workgroup per row.  Scores are mapped to order-preserving 32-bit keys;
// the k-th largest key is found by a most-significant-digit radix select
// (11 + 11 + 10 bits, LDS histograms, wave-level prefix sums on DPP), then one
// ordered pass emits every column above the threshold plus the first columns
// equal to it, in ascending column order.  Rows of up to kLdsCols columns are
// read from HBM once and kept in LDS as keys; longer rows are re-read (they
// stay in L2 / Infinity Cache between the passes).
#include "common.h"

namespace chipmunk {

constexpr int kLdsCols = 14208;  // 55.5 KB of keys + 8 KB histogram fit one 64 KB LDS allocation
constexpr int kBins = 2048;

__device__ __forceinline__ uint32_t score_key(float cur, const float* prev_ptr) {
    float s = cur;
    if (prev_ptr) s = fabsf(cur - *prev_ptr);
    if (s == 0.f) s = 0.f;  // -0 and +0 are the same score
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive prefix sum over the 64 lanes of a wave: DPP row shifts inside each
// row of 16 lanes, then the three lower rows' totals are added.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false);  // row_shr:8
    uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)v, 15);
    uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)v, 31);
    uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)v, 47);
    int row = (threadIdx.x & 63) >> 4;
    uint32_t add = (row > 0 ? t0 : 0u) + (row > 1 ? t1 : 0u) + (row > 2 ? t2 : 0u);
    return v + add;
}

// exclusive prefix sum of one value per thread over the 256 threads of the
// workgroup; *total receives the sum.  s_wave: 4 words of LDS.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* s_wave, uint32_t* total) {
    uint32_t inc = wave_inclusive_scan(v);
    int w = threadIdx.x >> 6;
    __syncthreads();  // s_wave may still be read by a previous call
    if ((threadIdx.x & 63) == 63) s_wave[w] = inc;
    __syncthreads();
    uint32_t w0 = s_wave[0], w1 = s_wave[1], w2 = s_wave[2], w3 = s_wave[3];
    uint32_t before = (w > 0 ? w0 : 0u) + (w > 1 ? w1 : 0u) + (w > 2 ? w2 : 0u);
    *total = w0 + w1 + w2 + w3;
    return before + inc - v;
}

template <bool LDS_ROW>
__global__ __launch_bounds__(256) void topk_cols_kernel(const float* __restrict__ cur,
                                                        const float* __restrict__ prev, int C, int64_t ld,
                                                        int k, int32_t* __restrict__ idx,
                                                        int32_t* __restrict__ counts, int k_stride) {
    __shared__ uint32_t s_hist[kBins];
    __shared__ uint32_t s_keys[LDS_ROW ? kLdsCols : 4];
    __shared__ uint32_t s_wave[4];
    __shared__ uint32_t s_pick[2];

    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    const float* crow = cur + row * ld;
    const float* prow = prev ? prev + row * ld : nullptr;
    int32_t* out = idx + row * (int64_t)k_stride;
    if (tid == 0) counts[row] = k;
    if (k == 0) return;

    const int C4 = (C + 3) >> 2;  // rows are read as 4-column groups (ld % 4 == 0 keeps them aligned)

    // keys of columns 4*j4 .. 4*j4+3; columns at or beyond C do not exist (valid = how many do)
    auto keys4 = [&](int j4, uint32_t (&key)[4]) -> int {
        int valid = min(4, C - 4 * j4);
        if (LDS_ROW) {
            uint4 kk = *reinterpret_cast<const uint4*>(&s_keys[4 * j4]);
            key[0] = kk.x; key[1] = kk.y; key[2] = kk.z; key[3] = kk.w;
        } else {
            float4 c4 = *reinterpret_cast<const float4*>(crow + 4 * j4);
            float cv[4] = {c4.x, c4.y, c4.z, c4.w};
            float pv[4] = {0.f, 0.f, 0.f, 0.f};
            if (prow) {
                float4 p4 = *reinterpret_cast<const float4*>(prow + 4 * j4);
                pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
            }
#pragma unroll
            for (int e = 0; e < 4; e++) key[e] = score_key(cv[e], prow ? &pv[e] : nullptr);
        }
        return valid;
    };

    if (LDS_ROW) {
        for (int j4 = tid; j4 < C4; j4 += 256) {
            float4 c4 = *reinterpret_cast<const float4*>(crow + 4 * j4);
            float cv[4] = {c4.x, c4.y, c4.z, c4.w};
            float pv[4] = {0.f, 0.f, 0.f, 0.f};
            if (prow) {
                float4 p4 = *reinterpret_cast<const float4*>(prow + 4 * j4);
                pv[0] = p4.x; pv[1] = p4.y; pv[2] = p4.z; pv[3] = p4.w;
            }
            uint4 kk;
            kk.x = score_key(cv[0], prow ? &pv[0] : nullptr);
            kk.y = score_key(cv[1], prow ? &pv[1] : nullptr);
            kk.z = score_key(cv[2], prow ? &pv[2] : nullptr);
            kk.w = score_key(cv[3], prow ? &pv[3] : nullptr);
            *reinterpret_cast<uint4*>(&s_keys[4 * j4]) = kk;
        }
    }

    // ---- radix select of the k-th largest key -------------------------------
    uint32_t known = 0;       // the digits fixed so far, in place
    uint32_t want = (uint32_t)k;  // rank still to be found among the keys that match `known`
    const int shifts[3] = {21, 10, 0};
    const int widths[3] = {11, 11, 10};
#pragma unroll 1
    for (int pass = 0; pass < 3; pass++) {
        const int shift = shifts[pass];
        const uint32_t digit_mask = (1u << widths[pass]) - 1u;
        const uint32_t hi_mask = pass == 0 ? 0u : ~((1u << (shift + widths[pass])) - 1u);
        for (int b = tid; b < kBins; b += 256) s_hist[b] = 0;
        __syncthreads();
        for (int j4 = tid; j4 < C4; j4 += 256) {
            uint32_t key[4];
            int valid = keys4(j4, key);
#pragma unroll
            for (int e = 0; e < 4; e++)
                if (e < valid && (key[e] & hi_mask) == known) atomicAdd(&s_hist[(key[e] >> shift) & digit_mask], 1u);
        }
        __syncthreads();
        // thread t owns the 8 bins 2047-8t .. 2040-8t (descending); find where the
        // count from the top reaches `want`
        uint32_t mine[8];
        uint32_t sum = 0;
#pragma unroll
        for (int e = 0; e < 8; e++) {
            mine[e] = s_hist[kBins - 1 - (8 * tid + e)];
            sum += mine[e];
        }
        uint32_t total;
        uint32_t above = block_exclusive_scan(sum, s_wave, &total);
        if (above < want && want <= above + sum) {
            uint32_t acc = above;
#pragma unroll
            for (int e = 0; e < 8; e++) {
                if (acc < want && want <= acc + mine[e]) {
                    s_pick[0] = (uint32_t)(kBins - 1 - (8 * tid + e));
                    s_pick[1] = want - acc;
                }
                acc += mine[e];
            }
        }
        __syncthreads();
        known |= s_pick[0] << shift;
        want = s_pick[1];
        __syncthreads();
    }
    const uint32_t thr = known;     // the k-th largest key
    const uint32_t take_eq = want;  // how many columns equal to it are kept (the lowest ones)

    // ---- ordered emission ---------------------------------------------------
    uint32_t run_gt = 0, run_eq = 0;
    for (int base4 = 0; base4 < C4; base4 += 256) {
        int j4 = base4 + tid;
        uint32_t key[4] = {0, 0, 0, 0};
        int valid = 0;
        if (j4 < C4) valid = keys4(j4, key);
        uint32_t ngt = 0, neq = 0;
#pragma unroll
        for (int e = 0; e < 4; e++) {
            if (e < valid) {
                ngt += key[e] > thr;
                neq += key[e] == thr;
            }
        }
        uint32_t total;
        uint32_t before = block_exclusive_scan(ngt | (neq << 16), s_wave, &total);
        uint32_t gt_before = run_gt + (before & 0xffffu);
        uint32_t eq_before = run_eq + (before >> 16);
#pragma unroll
        for (int e = 0; e < 4; e++) {
            if (e < valid) {
                bool gt = key[e] > thr, eq = key[e] == thr;
                if (gt || (eq && eq_before < take_eq)) out[gt_before + min(eq_before, take_eq)] = 4 * j4 + e;
                gt_before += gt;
                eq_before += eq;
            }
        }
        run_gt += total & 0xffffu;
        run_eq += total >> 16;
    }
}

}  // namespace chipmunk

using namespace chipmunk;

extern "C" int32_t chipmunk_topk_cols(const float* cur, const float* prev, int R, int C, int64_t ld, int k,
                                      int32_t* idx, int32_t* counts, int k_stride, void* stream) {
    if (!cur || !idx || !counts) return CHIPMUNK_ERR_NULL;
    if (R < 1 || C < 1 || ld < C || k < 0 || k > C || k_stride < k) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(cur) || !aligned16(prev) || (ld % 4) != 0 || (reinterpret_cast<uintptr_t>(idx) & 3u) ||
        (reinterpret_cast<uintptr_t>(counts) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    hipStream_t s = (hipStream_t)stream;
    if (C <= kLdsCols)
        hipLaunchKernelGGL((topk_cols_kernel<true>), dim3((unsigned)R), dim3(256), 0, s, cur, prev, C, ld, k, idx,
                           counts, k_stride);
    else
        hipLaunchKernelGGL((topk_cols_kernel<false>), dim3((unsigned)R), dim3(256), 0, s, cur, prev, C, ld, k, idx,
                           counts, k_stride);
    return launch_status();
}
