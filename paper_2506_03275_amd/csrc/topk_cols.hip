// Exact per-row top-k column selection (Sec. 3.3.1 idx = TopK_k(D); Alg. 7
// idx = TopK(|T - T_m|)) for gfx950.
//
// One workgroup per row.  Scores are mapped to order-preserving 32-bit keys.
// The k-th largest key (the threshold) is found by a most-significant-digit
// radix select (digits of up to 11 bits, LDS histograms, wave-level prefix
// sums on DPP); the selected columns are every column above the threshold plus
// the first columns equal to it, written in ascending column order.
//   - Rows of up to kLdsCols columns are read from HBM once and kept in LDS as
//     keys; every pass runs on LDS.
//   - Longer rows (the attention column sums, 10^5 columns) are read from HBM
//     once as well: two pivots taken from a 4096-score sample bracket the
//     threshold; the single pass over the row marks the columns above the
//     upper pivot in a bit mask in LDS and collects the few thousand scores
//     between the pivots; the exact threshold is selected among those, their
//     bits are added, and the indices are written from the mask.  If the
//     bracket misses (probability about 1e-3 per row), if the candidates
//     overflow (heavy ties) or if the mask would not fit LDS, the row falls
//     back to histogram passes over global memory: the result is exact in
//     every case.
#include "common.h"

#include <algorithm>

namespace chipmunk {

constexpr int kLdsCols = 14208;   // 55.5 KB of keys + 8 KB histogram fit one 64 KB LDS allocation
constexpr int kBins = 2048;
constexpr float kPivotSigmas = 3.5f;  // slack of the sample pivots around the threshold, in standard deviations

// key(a) > key(b) exactly when a > b; no finite or infinite score has key 0
__device__ __forceinline__ uint32_t key_of_score(float s) {
    if (s == 0.f) s = 0.f;  // -0 and +0 are the same score
    uint32_t u = __float_as_uint(s);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ float score_of_key(uint32_t key) {
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

__device__ __forceinline__ uint32_t score_key(float cur, float prev, bool has_prev) {
    return key_of_score(has_prev ? fabsf(cur - prev) : cur);
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

// The small shared arrays of the selection routines.
struct SelectScratch {
    uint32_t* hist;   // kBins words
    uint32_t* wave;   // 2 (NT / 64) words: two sets of per-wave totals used in turn.  A set is written again only
                      // after the barrier of the scan in between, which no thread passes before it has read
                      // the set: one barrier per scan is enough
    uint32_t* pick;   // 6 words
    int flip;         // which set the next scan uses (the same in every thread)
};

// exclusive prefix sum of one value per thread over the NT threads of the
// workgroup; *total receives the sum.
template <int NT>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, SelectScratch& sc, uint32_t* total) {
    constexpr int NW = NT / 64;
    uint32_t inc = wave_inclusive_scan(v);
    int w = threadIdx.x >> 6;
    uint32_t* set = sc.wave + sc.flip * NW;
    sc.flip ^= 1;
    if ((threadIdx.x & 63) == 63) set[w] = inc;
    __syncthreads();
    uint32_t before = 0, sum = 0;
#pragma unroll
    for (int i = 0; i < NW; i++) {
        const uint32_t wi = set[i];
        before += i < w ? wi : 0u;
        sum += wi;
    }
    *total = sum;
    return before + inc - v;
}

// Key sources hand out four consecutive keys per call in two steps, so that a caller
// can issue several loads before it consumes the first: load(j4) fetches group j4
// (clamped to the last group, hence always in bounds and free of branches), keys()
// turns what was loaded into keys and returns how many of the four exist (0 when j4
// lies past the end).

// A row in global memory.
template <bool HAS_PREV>
struct GlobalRowKeys {
    const float* cur;
    const float* prev;
    int C;
    struct Raw {
        float4 c, p;
    };
    __device__ __forceinline__ Raw load(int j4) const {
        const int j = min(j4, ((C + 3) >> 2) - 1);
        Raw r;
        r.c = *reinterpret_cast<const float4*>(cur + 4 * j);
        if constexpr (HAS_PREV)
            r.p = *reinterpret_cast<const float4*>(prev + 4 * j);
        else
            r.p = float4{0.f, 0.f, 0.f, 0.f};
        return r;
    }
    __device__ __forceinline__ int keys(const Raw& r, int j4, uint32_t (&key)[4]) const {
        key[0] = score_key(r.c.x, r.p.x, HAS_PREV);
        key[1] = score_key(r.c.y, r.p.y, HAS_PREV);
        key[2] = score_key(r.c.z, r.p.z, HAS_PREV);
        key[3] = score_key(r.c.w, r.p.w, HAS_PREV);
        return max(0, min(4, C - 4 * j4));
    }
};

// Keys already in LDS (a whole short row, a sample, or the candidates of a long row).
struct LdsKeys {
    const uint32_t* data;
    int n;
    typedef uint4 Raw;
    __device__ __forceinline__ Raw load(int j4) const {
        return *reinterpret_cast<const uint4*>(data + 4 * min(j4, ((n + 3) >> 2) - 1));
    }
    __device__ __forceinline__ int keys(const Raw& r, int j4, uint32_t (&key)[4]) const {
        key[0] = r.x; key[1] = r.y; key[2] = r.z; key[3] = r.w;
        return max(0, min(4, n - 4 * j4));
    }
};

// One radix digit: hist[d] = how many of the n keys behind `src` agree with `known`
// on the bits selected by hi_mask and have digit d = (key >> shift) & digit_mask.
// Nobody reads hist when this is called (every reader below ends with a barrier).
template <int NT, typename Src>
__device__ __forceinline__ void digit_histogram(const Src& src, int n, uint32_t known, uint32_t hi_mask, int shift,
                                                uint32_t digit_mask, uint32_t* hist) {
    const int tid = threadIdx.x;
    const int n4 = (n + 3) >> 2;
    for (int b = tid; b < kBins; b += NT) hist[b] = 0;
    __syncthreads();
    for (int j4 = tid; j4 < n4; j4 += 2 * NT) {
        typename Src::Raw raw0 = src.load(j4), raw1 = src.load(j4 + NT);
        uint32_t key[2][4];
        int valid[2];
        valid[0] = src.keys(raw0, j4, key[0]);
        valid[1] = src.keys(raw1, j4 + NT, key[1]);
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int e = 0; e < 4; e++)
                if (e < valid[h] && (key[h][e] & hi_mask) == known)
                    atomicAdd(&hist[(key[h][e] >> shift) & digit_mask], 1u);
    }
    __syncthreads();
}

// For each of NQ ranks (1-based, counted from the highest digit down): the digit whose
// bin holds that rank, the rank inside the bin, and how many keys the bin holds.
// Ends with a barrier behind which nobody reads hist or sc.pick's previous contents any more.
template <int NT, int NQ>
__device__ __forceinline__ void pick_digits(const uint32_t (&want)[NQ], const uint32_t* hist, SelectScratch& sc,
                                            uint32_t (&digit)[NQ], uint32_t (&rest)[NQ], uint32_t (&held)[NQ]) {
    const int tid = threadIdx.x;
    constexpr int PER = kBins / NT;   // thread t owns the bins 2047 - PER t .. (descending)
    uint32_t mine[PER];
    uint32_t sum = 0;
#pragma unroll
    for (int e = 0; e < PER; e++) {
        mine[e] = hist[kBins - 1 - (PER * tid + e)];
        sum += mine[e];
    }
    uint32_t total;
    const uint32_t above = block_exclusive_scan<NT>(sum, sc, &total);
#pragma unroll
    for (int q = 0; q < NQ; q++) {
        if (above < want[q] && want[q] <= above + sum) {
            uint32_t acc = above;
#pragma unroll
            for (int e = 0; e < PER; e++) {
                if (acc < want[q] && want[q] <= acc + mine[e]) {
                    sc.pick[3 * q] = (uint32_t)(kBins - 1 - (PER * tid + e));
                    sc.pick[3 * q + 1] = want[q] - acc;
                    sc.pick[3 * q + 2] = mine[e];
                }
                acc += mine[e];
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < NQ; q++) {
        digit[q] = sc.pick[3 * q];
        rest[q] = sc.pick[3 * q + 1];
        held[q] = sc.pick[3 * q + 2];
    }
}

// Radix select: the `rank`-th largest (1-based) among those of the n keys behind `src`
// that agree with `known` above bit `low_bits`.  Digits of up to 11 bits are resolved
// from bit low_bits down to bit stop_bits; the result is the selected key with the bits
// below stop_bits cleared, and *take_eq receives the rank left inside the last bin (with
// stop_bits = 0: how many keys equal to the result rank at or above it).
// Called by all NT threads.
template <int NT, typename Src>
__device__ __forceinline__ uint32_t radix_select(const Src& src, int n, uint32_t rank, SelectScratch& sc,
                                                 uint32_t* take_eq, uint32_t known = 0, int low_bits = 32,
                                                 int stop_bits = 0) {
    uint32_t want[1] = {rank};
    int remaining = low_bits;
#pragma unroll 1
    while (remaining > stop_bits) {
        const int width = min(11, remaining);
        const int shift = remaining - width;
        const uint32_t hi_mask = remaining >= 32 ? 0u : ~((1u << remaining) - 1u);
        digit_histogram<NT>(src, n, known, hi_mask, shift, (1u << width) - 1u, sc.hist);
        uint32_t digit[1], held[1];
        pick_digits<NT, 1>(want, sc.hist, sc, digit, want, held);
        known |= digit[0] << shift;
        remaining = shift;
    }
    *take_eq = want[0];
    return known;
}

// Ordered emission: every column whose key exceeds thr, and the first take_eq
// columns whose key equals it, in ascending column order.  One iteration covers
// 16 NT columns: wave w owns columns [1024 w, 1024 w + 1024) of them as four
// coalesced groups of 256, so one cross-wave exchange serves 16 keys per thread.
template <int NT, typename Src>
__device__ __forceinline__ void emit_selected(const Src& src, int C, uint32_t thr, uint32_t take_eq,
                                              int32_t* __restrict__ out, SelectScratch& sc) {
    constexpr int U = 4;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int C4 = (C + 3) >> 2;
    uint32_t run_gt = 0, run_eq = 0;
    for (int base4 = 0; base4 < C4; base4 += NT * U) {
        uint32_t key[U][4];
        int valid[U], j4[U];
        typename Src::Raw raw[U];
#pragma unroll
        for (int u = 0; u < U; u++) {
            j4[u] = base4 + w * (64 * U) + u * 64 + lane;
            raw[u] = src.load(j4[u]);
        }
#pragma unroll
        for (int u = 0; u < U; u++) valid[u] = src.keys(raw[u], j4[u], key[u]);
        uint32_t cnt[U], inc[U], tot[U], wave_sum = 0;
#pragma unroll
        for (int u = 0; u < U; u++) {
            uint32_t ngt = 0, neq = 0;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                if (e < valid[u]) {
                    ngt += key[u][e] > thr;
                    neq += key[u][e] == thr;
                }
            }
            cnt[u] = ngt | (neq << 16);
            inc[u] = wave_inclusive_scan(cnt[u]);
            tot[u] = (uint32_t)__builtin_amdgcn_readlane((int)inc[u], 63);
            wave_sum += tot[u];
        }
        uint32_t* set = sc.wave + sc.flip * (NT / 64);
        sc.flip ^= 1;
        if (lane == 0) set[w] = wave_sum;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int i = 0; i < NT / 64; i++) {
            const uint32_t wi = set[i];
            before += i < w ? wi : 0u;
            total += wi;
        }
#pragma unroll
        for (int u = 0; u < U; u++) {
            uint32_t mine = before + inc[u] - cnt[u];
            uint32_t gt_before = run_gt + (mine & 0xffffu);
            uint32_t eq_before = run_eq + (mine >> 16);
#pragma unroll
            for (int e = 0; e < 4; e++) {
                if (e < valid[u]) {
                    bool gt = key[u][e] > thr, eq = key[u][e] == thr;
                    if (gt || (eq && eq_before < take_eq)) out[gt_before + min(eq_before, take_eq)] = 4 * j4[u] + e;
                    gt_before += gt;
                    eq_before += eq;
                }
            }
            before += tot[u];
        }
        run_gt += total & 0xffffu;
        run_eq += total >> 16;
    }
}

// Rows that fit LDS.
template <bool HAS_PREV>
__global__ __launch_bounds__(256) void topk_short_rows_kernel(const float* __restrict__ cur,
                                                              const float* __restrict__ prev, int C, int64_t ld,
                                                              int k, int32_t* __restrict__ idx,
                                                              int32_t* __restrict__ counts, int k_stride) {
    // dynamic LDS, sized to the row so that short rows leave room for more workgroups per CU:
    // kBins + 16 words, then the row's keys (a multiple of four)
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    SelectScratch sc{smem, smem + kBins, smem + kBins + 8, 0};
    uint32_t* s_keys = smem + kBins + 16;
    const int tid = threadIdx.x;
    const int64_t row = blockIdx.x;
    if (tid == 0) counts[row] = k;
    if (k == 0) return;
    GlobalRowKeys<HAS_PREV> g{cur + row * ld, HAS_PREV ? prev + row * ld : nullptr, C};
    const int C4 = (C + 3) >> 2;
    constexpr int U = 4;
    for (int base4 = 0; base4 < C4; base4 += 256 * U) {
        typename GlobalRowKeys<HAS_PREV>::Raw raw[U];
#pragma unroll
        for (int u = 0; u < U; u++) raw[u] = g.load(base4 + u * 256 + tid);
#pragma unroll
        for (int u = 0; u < U; u++) {
            const int j4 = base4 + u * 256 + tid;
            uint32_t key[4];
            if (g.keys(raw[u], j4, key) > 0)
                *reinterpret_cast<uint4*>(&s_keys[4 * j4]) = uint4{key[0], key[1], key[2], key[3]};
        }
    }
    LdsKeys src{s_keys, C};
    uint32_t take_eq;
    uint32_t thr = radix_select<256>(src, C, (uint32_t)k, sc, &take_eq);
    emit_selected<256>(src, C, thr, take_eq, idx + row * (int64_t)k_stride, sc);
}

// The candidates of a long row are (key, column) pairs.  Their keys:
struct CandidateKeys {
    const uint2* pairs;
    int n;
    struct Raw {
        uint4 a, b;   // pairs 4 j4, 4 j4 + 1 and 4 j4 + 2, 4 j4 + 3
    };
    __device__ __forceinline__ Raw load(int j4) const {
        const uint4* at = reinterpret_cast<const uint4*>(pairs + 4 * min(j4, ((n + 3) >> 2) - 1));
        return Raw{at[0], at[1]};
    }
    __device__ __forceinline__ int keys(const Raw& r, int j4, uint32_t (&key)[4]) const {
        key[0] = r.a.x; key[1] = r.a.z; key[2] = r.b.x; key[3] = r.b.z;
        return max(0, min(4, n - 4 * j4));
    }
};

// Those whose key equals the threshold, keyed so that the lower column ranks higher.
struct CandidateTieKeys {
    const uint2* pairs;
    int n;
    uint32_t thr;
    typedef CandidateKeys::Raw Raw;
    __device__ __forceinline__ Raw load(int j4) const { return CandidateKeys{pairs, n}.load(j4); }
    __device__ __forceinline__ int keys(const Raw& r, int j4, uint32_t (&key)[4]) const {
        key[0] = r.a.x == thr ? ~r.a.y : 0u;
        key[1] = r.a.z == thr ? ~r.a.w : 0u;
        key[2] = r.b.x == thr ? ~r.b.y : 0u;
        key[3] = r.b.z == thr ? ~r.b.w : 0u;
        return max(0, min(4, n - 4 * j4));
    }
};

constexpr int kLongThreads = 512;              // threads of a workgroup of the long-row kernel
constexpr int kLongWaves = kLongThreads / 64;
constexpr int kLongSmall = 48;                 // words of small shared arrays behind the histogram
constexpr uint32_t kCrowdedBin = 16;           // sample keys in a pivot's bin beyond which the bin is resolved further

// State of one wave during the single pass over a long row.
struct LongRowPass {
    float f_hi, f_lo;         // the pivots, as scores (never NaN; f_lo <= f_hi)
    uint32_t* s_mask;         // one bit per column: bit (col & 31) of word col >> 5; zero before the pass
    uint2* s_cand;            // this wave's candidates: (raw bits of the score, column)
    uint32_t seg_cap;         // slots in this wave's candidate segment
    uint32_t slot;            // candidates appended so far (the same in every lane)
    uint32_t n_above;         // per lane: mask bits this lane has set
    uint32_t bit[4];          // the lane's four bits inside its mask word: 1 << (4 (lane % 8) + e)
    int C, G;                 // columns; groups of 256 columns
};

// Appends the scores of the lanes named by `who` (`mine`: this lane is one of them) to the wave's candidates.
__device__ __forceinline__ void long_row_append(LongRowPass& st, uint64_t who, bool mine, float score, int col) {
    uint32_t pos = __builtin_amdgcn_mbcnt_hi((uint32_t)(who >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)who, st.slot));
    pos = min(pos, st.seg_cap - 1u);  // an overflow is detected from the count
    if (mine) st.s_cand[pos] = uint2{__float_as_uint(score), (uint32_t)col};
    st.slot += (uint32_t)__builtin_popcountll(who);
}

// One group of 256 columns: lane l holds the scores of columns 256 g + 4 l .. + 3.  Its four "above the upper
// pivot" bits are OR-ed into mask word 8 g + l / 8 by an LDS atomic; scores between the pivots are appended to
// the wave's candidates.  About one score in fifty is a candidate, so a lane rarely has more than one: the first
// candidate of every lane goes out in one step, further ones (some lane of the wave has one in about one group
// out of six) in a step per element.  The order of the candidates does not matter.
// The pass is bound by the number of vector and of scalar instructions a wave issues per group (a compute unit
// runs out of issue slots before it runs out of memory bandwidth), hence the care: "between the pivots" is one
// comparison (the median of score and pivots is the score), so that its lane mask is used as it comes, and lane
// masks are combined as scalars.
template <bool MASKED>
__device__ __forceinline__ void long_row_group(LongRowPass& st, const float (&s)[4], int g, int lane) {
    const int col0 = (g * 64 + lane) * 4;
    bool between[4];
    uint64_t cand[4];
    uint32_t word = 0;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        bool above = s[e] > st.f_hi;
        between[e] = __builtin_amdgcn_fmed3f(s[e], st.f_lo, st.f_hi) == s[e];   // f_lo <= s <= f_hi
        if (MASKED) {
            const bool exists = col0 + e < st.C;
            above = above && exists;
            between[e] = between[e] && exists;
        }
        word |= above ? st.bit[e] : 0u;
        cand[e] = __builtin_amdgcn_ballot_w64(between[e]);
    }
    if (!MASKED || g < st.G) atomicOr(&st.s_mask[g * 8 + (lane >> 3)], word);
    st.n_above += __popc(word);
    const uint64_t upto1 = cand[0] | cand[1], upto2 = upto1 | cand[2], any = upto2 | cand[3];
    if (any != 0) {
        const float first = between[0] ? s[0] : between[1] ? s[1] : between[2] ? s[2] : s[3];
        const int first_e = between[0] ? 0 : between[1] ? 1 : between[2] ? 2 : 3;
        long_row_append(st, any, between[0] || between[1] || between[2] || between[3], first, col0 + first_e);
        const uint64_t more1 = cand[1] & cand[0], more2 = cand[2] & upto1, more3 = cand[3] & upto2;
        if ((more1 | more2 | more3) != 0) {
            if (more1 != 0) long_row_append(st, more1, between[1] && between[0], s[1], col0 + 1);
            if (more2 != 0) long_row_append(st, more2, between[2] && (between[0] || between[1]), s[2], col0 + 2);
            if (more3 != 0)
                long_row_append(st, more3, between[3] && (between[0] || between[1] || between[2]), s[3], col0 + 3);
        }
    }
}

// Where the threshold is expected among S sampled keys: a rank that very likely lies
// above it and one that very likely lies below it (1-based from the top; the first may
// be < 1 and the second > S, which stand for "no such sample").
__host__ __device__ inline void pivot_ranks(int k, int C, int S, int* rank_hi, int* rank_lo) {
    const float q = (float)k / (float)C;
    const float r = q * (float)S;
    const float margin = kPivotSigmas * sqrtf(fmaxf((float)S * q * (1.f - q), 1.f)) + 2.f;
    *rank_hi = (int)floorf(r - margin);
    *rank_lo = (int)ceilf(r + margin) + 1;
}

// Rows too long for LDS; eight waves per row.  With BRACKET the row is read from HBM once:
//   1. S scores are sampled as segments of 16 consecutive columns; two pivots that bracket
//      the threshold with 3.5 standard deviations of slack are selected from the sample;
//   2. one pass over the row records, as a bit per column in LDS, which scores exceed
//      the upper pivot, and appends the (score, column) pairs between the pivots to LDS
//      (each wave to a segment of seg_cap slots of its own, so that no atomics are needed);
//   3. the exact threshold is selected among those candidates and their bits are set;
//   4. the column indices are written from the bit mask in ascending order.
// If the bracket misses the threshold or the candidates overflow, or without BRACKET
// (rows whose mask would not fit LDS), the threshold is selected by three histogram
// passes over the row in global memory and a fourth pass writes the indices.
// A wave alone needs about 600 cycles per 256 columns of the pass (its instructions issue in order), far more
// than the memory system does, so the row is spread over eight waves; LDS allows three rows per CU.
// Dynamic LDS: kBins + kLongSmall words, and with BRACKET 2 kLongWaves seg_cap + 8 ceil(C / 256) more.
template <bool BRACKET, bool HAS_PREV, int S>
__global__ __launch_bounds__(kLongThreads, 6) void topk_long_rows_kernel(const float* __restrict__ cur,
                                                                      const float* __restrict__ prev, int C, int64_t ld,
                                                                      int k, int32_t* __restrict__ idx,
                                                                      int32_t* __restrict__ counts, int k_stride,
                                                                      int seg_cap) {
    constexpr int NT = kLongThreads, NW = kLongWaves;
    extern __shared__ __attribute__((aligned(16))) uint32_t smem[];
    SelectScratch sc{smem, smem + kBins, smem + kBins + 2 * NW, 0};   // hist, two sets of NW scan words, 6 pick words
    uint32_t* s_seg = sc.pick + 6;          // NW: candidates appended by each wave
    uint32_t* s_above = s_seg + NW;         // 1: scores above the upper pivot
    uint32_t* s_range = s_above + 1;        // 2 NW: every wave's smallest and largest sample key
    static_assert(5 * NW + 7 <= kLongSmall, "the small arrays fit their words");
    uint2* s_cand = reinterpret_cast<uint2*>(smem + kBins + kLongSmall);  // NW seg_cap candidates: (score, later key;
                                                                          // column); a second histogram before that
    uint32_t* s_mask = smem + kBins + kLongSmall + 2 * NW * seg_cap;      // one bit per column
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row = blockIdx.x;
    if (tid == 0) counts[row] = k;
    if (k == 0) return;
    typedef GlobalRowKeys<HAS_PREV> Row;
    Row g{cur + row * ld, HAS_PREV ? prev + row * ld : nullptr, C};
    const int C4 = (C + 3) >> 2;
    int32_t* out = idx + row * (int64_t)k_stride;

    if constexpr (BRACKET) {
        // ---- 1. pivots from a sample ---------------------------------------------------------
        // Thread t < S / 16 holds segment t of the sample as 16 keys in registers; the sample never goes to LDS.
        // While the loads are in flight: both histograms and the column mask are cleared.
        constexpr int kSegments = S / 16;
        static_assert(kSegments <= NT, "one segment per thread at most");
        static_assert(2 * NW * 128 >= kBins, "the second histogram fits the smallest candidate area (seg_cap >= 128)");
        const bool have = tid < kSegments;
        const int G = (C4 + 63) >> 6;
        uint32_t* hist2 = reinterpret_cast<uint32_t*>(s_cand);   // free until the pass
        // the pass's batches (step 2): U groups of 256 columns each
        constexpr int U = HAS_PREV ? 2 : 4;
        const int full4 = C >> 2;                      // float4 groups that exist completely
        const int full_batches = full4 / (64 * U);
        const int last_safe4 = full4 - 64 * U;         // last start from which a whole batch is in bounds
        const float4* cur4 = reinterpret_cast<const float4*>(g.cur);
        const float4* prev4 = reinterpret_cast<const float4*>(g.prev);
        float4 rc[U], rp[U];
        int b = w;
        uint32_t skey[16];
        {
            typename Row::Raw raw[4];
            const int start4 = (int)(((int64_t)min(tid, kSegments - 1) * C) / kSegments) >> 4 << 2;  // 16 | column
#pragma unroll
            for (int v = 0; v < 4; v++) raw[v] = g.load(start4 + v);
            {   // the wave's first batch of the pass is requested behind the sample: it lands while the pivots are found
                const int at = min(b * 64 * U, last_safe4);
#pragma unroll
                for (int u = 0; u < U; u++) {
                    rc[u] = cur4[at + u * 64 + lane];
                    if constexpr (HAS_PREV) rp[u] = prev4[at + u * 64 + lane];
                }
            }
            for (int i = tid; i < kBins / 4; i += NT) {
                reinterpret_cast<uint4*>(sc.hist)[i] = uint4{0u, 0u, 0u, 0u};
                reinterpret_cast<uint4*>(hist2)[i] = uint4{0u, 0u, 0u, 0u};
            }
            for (int i = tid; i < 2 * G; i += NT) reinterpret_cast<uint4*>(s_mask)[i] = uint4{0u, 0u, 0u, 0u};
            if (tid == 0) *s_above = 0;
#pragma unroll
            for (int v = 0; v < 4; v++) {
                uint32_t key[4];
                g.keys(raw[v], start4 + v, key);
#pragma unroll
                for (int e = 0; e < 4; e++) skey[4 * v + e] = key[e];
            }
        }
        // The sample's keys agree on their leading bits (scores of one row share sign and, mostly, exponent); the
        // digits are taken below that common prefix, where the keys spread over the bins (digits of the leading
        // bits would send a whole wave's atomics to a handful of bins).
        uint32_t kmin = 0xffffffffu, kmax = 0u;
        if (have) {
#pragma unroll
            for (int j = 0; j < 16; j++) {
                kmin = min(kmin, skey[j]);
                kmax = max(kmax, skey[j]);
            }
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            kmin = min(kmin, (uint32_t)__shfl_xor((int)kmin, off));
            kmax = max(kmax, (uint32_t)__shfl_xor((int)kmax, off));
        }
        if (lane == 0) {
            s_range[w] = kmin;
            s_range[NW + w] = kmax;
        }
        __syncthreads();   // also: histograms and mask are clear
#pragma unroll
        for (int i = 0; i < NW; i++) {
            kmin = min(kmin, s_range[i]);
            kmax = max(kmax, s_range[NW + i]);
        }
        int remaining = 32 - __clz((int)(kmin ^ kmax));          // bits in which the sample's keys can differ
        if (kmin == kmax) remaining = 0;
        const uint32_t prefix = remaining >= 32 ? 0u : (kmin >> remaining) << remaining;

        int rank_hi, rank_lo;
        pivot_ranks(k, C, S, &rank_hi, &rank_lo);
        // Both ranks are resolved (clamped into the sample); a pivot whose rank lies outside is replaced below.
        uint32_t want[2] = {(uint32_t)max(rank_hi, 1), (uint32_t)min(rank_lo, S)}, digit[2], held[2];
        uint32_t key_hi = prefix, key_lo = prefix;
        int unresolved = remaining;                               // low bits of the pivots not resolved
        auto sample_histogram = [&](uint32_t* hist, uint32_t known, int above_bit, int shift, uint32_t digit_mask) {
            // keys that agree with `known` above bit `above_bit`
            if (have) {
#pragma unroll
                for (int j = 0; j < 16; j++)
                    if (above_bit >= 32 || (skey[j] >> above_bit) == (known >> above_bit))
                        atomicAdd(&hist[(skey[j] >> shift) & digit_mask], 1u);
            }
            __syncthreads();
        };
        if (remaining > 0) {
            const int width = min(11, remaining), shift = remaining - width;
            sample_histogram(sc.hist, prefix, 32, shift, (1u << width) - 1u);
            pick_digits<NT, 2>(want, sc.hist, sc, digit, want, held);
            key_hi |= digit[0] << shift;
            key_lo |= digit[1] << shift;
            unresolved = shift;
            // A bin that holds few sample keys is pivot enough (its upper or lower edge); a crowded one, as the
            // bins of a heavy-tailed row are, is resolved by a second digit.
            if (shift > 0 && (held[0] > kCrowdedBin || held[1] > kCrowdedBin)) {
                const int width2 = min(11, shift), shift2 = shift - width2;
                const uint32_t mask2 = (1u << width2) - 1u;
                if (digit[0] == digit[1]) {
                    sample_histogram(hist2, key_hi, shift, shift2, mask2);
                    pick_digits<NT, 2>(want, hist2, sc, digit, want, held);
                    key_hi |= digit[0] << shift2;
                    key_lo |= digit[1] << shift2;
                } else {
                    // the first histogram is free again behind the barrier that ended pick_digits
                    for (int i = tid; i < kBins / 4; i += NT) reinterpret_cast<uint4*>(sc.hist)[i] = uint4{0u, 0u, 0u, 0u};
                    uint32_t one[1] = {want[0]}, d[1], h[1];
                    sample_histogram(hist2, key_hi, shift, shift2, mask2);   // its barrier also covers the clearing
                    pick_digits<NT, 1>(one, hist2, sc, d, one, h);
                    key_hi |= d[0] << shift2;
                    one[0] = want[1];
                    sample_histogram(sc.hist, key_lo, shift, shift2, mask2);
                    pick_digits<NT, 1>(one, sc.hist, sc, d, one, h);
                    key_lo |= d[0] << shift2;
                }
                unresolved = shift2;
            }
        }
        uint32_t pivot_hi = key_hi | (unresolved >= 32 ? 0xffffffffu : (1u << unresolved) - 1u);
        uint32_t pivot_lo = key_lo;
        uint32_t unused;
        // widened to the keys of -infinity and +infinity at most: as scores, neither pivot is a NaN
        if (rank_hi < 1) pivot_hi = 0xff800000u;
        if (rank_lo > S) pivot_lo = 0x007fffffu;
        pivot_lo = max(pivot_lo, 0x007fffffu);
        pivot_hi = min(pivot_hi, 0xff800000u);

        // ---- 2. one pass over the row ----------------------------------------------------------
        // A batch is U groups of 256 columns; wave w takes batches w, w + NW, ...  The loads of the
        // next batch are issued before the current one is consumed.  Batches whose columns all
        // exist take the unmasked path; the one batch that holds the end of the row is masked.
        // (the second histogram, in the candidates' place, is dead: pick_digits ended with a barrier)
        LongRowPass st{score_of_key(pivot_hi), score_of_key(pivot_lo), s_mask, s_cand + w * seg_cap,
                       (uint32_t)seg_cap, 0u, 0u,
                       {1u << (4 * (lane & 7)), 2u << (4 * (lane & 7)), 4u << (4 * (lane & 7)), 8u << (4 * (lane & 7))},
                       C, G};
        for (; b < full_batches; b += NW) {
            float s[U][4];
#pragma unroll
            for (int u = 0; u < U; u++) {
                if constexpr (HAS_PREV) {
                    s[u][0] = fabsf(rc[u].x - rp[u].x); s[u][1] = fabsf(rc[u].y - rp[u].y);
                    s[u][2] = fabsf(rc[u].z - rp[u].z); s[u][3] = fabsf(rc[u].w - rp[u].w);
                } else {
                    s[u][0] = rc[u].x; s[u][1] = rc[u].y; s[u][2] = rc[u].z; s[u][3] = rc[u].w;
                }
            }
            const int at = min((b + NW) * 64 * U, last_safe4);
#pragma unroll
            for (int u = 0; u < U; u++) {
                rc[u] = cur4[at + u * 64 + lane];
                if constexpr (HAS_PREV) rp[u] = prev4[at + u * 64 + lane];
            }
#pragma unroll
            for (int u = 0; u < U; u++) long_row_group<false>(st, s[u], b * U + u, lane);
        }
        if (b == full_batches && b * U < G) {
#pragma unroll
            for (int u = 0; u < U; u++) {
                typename Row::Raw raw = g.load((b * U + u) * 64 + lane);  // clamped to the last group
                float s[4];
                if constexpr (HAS_PREV) {
                    s[0] = fabsf(raw.c.x - raw.p.x); s[1] = fabsf(raw.c.y - raw.p.y);
                    s[2] = fabsf(raw.c.z - raw.p.z); s[3] = fabsf(raw.c.w - raw.p.w);
                } else {
                    s[0] = raw.c.x; s[1] = raw.c.y; s[2] = raw.c.z; s[3] = raw.c.w;
                }
                long_row_group<true>(st, s, b * U + u, lane);
            }
        }
        if (lane == 0) s_seg[w] = st.slot;
        {
            const uint32_t wave_above = (uint32_t)__builtin_amdgcn_readlane((int)wave_inclusive_scan(st.n_above), 63);
            if (lane == 0 && wave_above != 0) atomicAdd(s_above, wave_above);
        }
        __syncthreads();
        uint32_t n_cand = 0, seg_max = 0;
#pragma unroll
        for (int i = 0; i < NW; i++) {
            const uint32_t used = s_seg[i];
            n_cand += used;
            seg_max = max(seg_max, used);
        }
        const uint32_t n_above = *s_above;
        const bool fits = seg_max <= (uint32_t)seg_cap;

        if (fits && n_above < (uint32_t)k && (uint32_t)k <= n_above + n_cand) {
            // ---- 3. exact threshold among the candidates; set the bits of the selected ones --------
            // Scores become keys relative to the lower pivot, 1 .. span + 1, which need few digits;
            // the unused slots of every segment get key 0, below every candidate.
            const int n_slots = NW * seg_cap;
            {
                const uint32_t used = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_seg[w]);
                for (uint32_t i = lane; i < (uint32_t)seg_cap; i += 64) {
                    uint32_t* slot = &st.s_cand[i].x;
                    *slot = i < used ? key_of_score(__uint_as_float(*slot)) - pivot_lo + 1u : 0u;
                }
            }
            const int low_bits = 32 - __clz((int)(pivot_hi - pivot_lo + 1u));
            uint32_t take_eq;
            CandidateKeys cand{s_cand, n_slots};
            const uint32_t thr = radix_select<NT>(cand, n_slots, (uint32_t)k - n_above, sc, &take_eq, 0u, low_bits);
            // candidates above the threshold are selected, and so are those equal to it unless there
            // are more of them than take_eq
            uint32_t n_eq = 0;
            for (int i = tid; i < n_slots; i += NT) {
                const uint2 kc = s_cand[i];
                if (kc.x >= thr) atomicOr(&s_mask[kc.y >> 5], 1u << (kc.y & 31));
                n_eq += kc.x == thr;
            }
            uint32_t n_eq_total;
            block_exclusive_scan<NT>(n_eq, sc, &n_eq_total);
            if (n_eq_total != take_eq) {
                // ties across the threshold: only the take_eq lowest columns among the equal ones stay
                CandidateTieKeys ties{s_cand, n_slots, thr};
                const uint32_t tie_key = radix_select<NT>(ties, n_slots, take_eq, sc, &unused);
                for (int i = tid; i < n_slots; i += NT) {
                    const uint2 kc = s_cand[i];
                    if (kc.x == thr && ~kc.y < tie_key) atomicAnd(&s_mask[kc.y >> 5], ~(1u << (kc.y & 31)));
                }
            }
            __syncthreads();

            // ---- 4. indices from the mask, ascending -----------------------------------------------
            // Wave v owns one share of the mask words; per step its lanes take 64 consecutive words,
            // so neighbouring lanes write neighbouring output slots.
            const int n_words = 8 * G;
            const int share = (n_words + NW - 1) / NW;
            const int q_begin = min(n_words, w * share), q_end = min(n_words, q_begin + share);
            uint32_t mine = 0;
            for (int wi = q_begin + lane; wi < q_end; wi += 64) mine += __popc(s_mask[wi]);
            uint32_t total;
            const uint32_t wave_base =
                block_exclusive_scan<NT>(mine, sc, &total) - (wave_inclusive_scan(mine) - mine);
            uint32_t base = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_base);
            // The indices of a step go through LDS (the wave's candidate segment, dead by now), so that they leave
            // as runs of 64 consecutive words per store instead of one scattered word per lane and set bit.
            uint32_t* stage = reinterpret_cast<uint32_t*>(s_cand + w * seg_cap);
            const uint32_t stage_cap = 2u * (uint32_t)seg_cap;
            for (int w0 = q_begin; w0 < q_end; w0 += 64) {
                const int wi = w0 + lane;
                uint32_t m = wi < q_end ? s_mask[wi] : 0u;
                const uint32_t inc = wave_inclusive_scan(__popc(m));
                const uint32_t step_total = (uint32_t)__builtin_amdgcn_readlane((int)inc, 63);
                uint32_t pos = inc - __popc(m);
                if (step_total <= stage_cap) {
                    while (m) {
                        stage[pos++] = wi * 32 + __ffs((int)m) - 1;
                        m &= m - 1;
                    }
                    // the wave's LDS accesses complete in order; only the compiler has to keep these apart
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    for (uint32_t i = lane; i < step_total; i += 64)
                        if (base + i < (uint32_t)k) out[base + i] = (int32_t)stage[i];
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                } else {   // a step that selects more than the segment holds: straight to memory
                    pos += base;
                    while (m) {
                        if (pos < (uint32_t)k) out[pos] = wi * 32 + __ffs((int)m) - 1;
                        pos++;
                        m &= m - 1;
                    }
                }
                base += step_total;
            }
            return;
        }
    }
    uint32_t take_eq;
    __syncthreads();  // whatever the single-pass attempt left in flight in LDS is over
    const uint32_t thr = radix_select<NT>(g, C, (uint32_t)k, sc, &take_eq);
    emit_selected<NT>(g, C, thr, take_eq, out, sc);
}

constexpr size_t kMaxLdsBytes = 160 * 1024;

// Launch shape of the single-pass kernel for rows of C columns of which k are kept: the
// sample size and the candidate slots per wave (1.3 times the expected number plus slack,
// as far as LDS allows, and no more than lets three rows share a CU's LDS when that is enough for the slack).
// Returns false when the column mask leaves no room for candidates.
struct LongRowPlan {
    int sample, seg_cap;
    size_t lds_bytes;
};

inline bool plan_long_rows(int C, int k, LongRowPlan* plan) {
    const int S = C >= 65536 ? 8192 : 4096;
    const size_t mask_words = 8 * (size_t)((C + 255) / 256);
    const size_t fixed_words = kBins + kLongSmall;
    const size_t per_cap = 2 * kLongWaves;        // LDS words per slot of every wave's segment (score and column)
    if ((fixed_words + mask_words + per_cap * 64) * 4 > kMaxLdsBytes) return false;
    int rank_hi, rank_lo;
    pivot_ranks(k, C, S, &rank_hi, &rank_lo);
    const double bracket = (double)(std::min(rank_lo, S + 1) - std::max(rank_hi, 0) + 1) / (double)S;
    const double expected = bracket * (double)C / kLongWaves;      // candidates per wave
    const size_t room = (kMaxLdsBytes / 4 - fixed_words - mask_words) / per_cap;
    const size_t room3 = kMaxLdsBytes / 4 / 3 > fixed_words + mask_words
                             ? (kMaxLdsBytes / 4 / 3 - fixed_words - mask_words) / per_cap : 0;   // three rows per CU
    size_t seg_cap = std::max((size_t)(expected * 1.3) + 96, (size_t)128);
    if (seg_cap > room3 && (double)room3 >= expected * 1.15 + 64) seg_cap = room3;
    seg_cap = std::min(std::min(seg_cap, room), (size_t)4096) / 16 * 16;
    plan->sample = S;
    plan->seg_cap = (int)seg_cap;
    plan->lds_bytes = (fixed_words + per_cap * seg_cap + mask_words) * 4;
    return seg_cap >= 128;   // the second histogram of the sample phase lies in the candidates' place
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
    const dim3 grid((unsigned)R), block(256), block_long(kLongThreads);
    LongRowPlan plan;
    if (C <= kLdsCols) {
        auto kernel = prev ? topk_short_rows_kernel<true> : topk_short_rows_kernel<false>;
        const size_t lds = (kBins + 16 + (size_t)((C + 3) / 4) * 4) * sizeof(uint32_t);
        hipLaunchKernelGGL(kernel, grid, block, lds, s, cur, prev, C, ld, k, idx, counts, k_stride);
    } else if (plan_long_rows(C, k, &plan)) {
        auto kernel = plan.sample == 8192
                          ? (prev ? topk_long_rows_kernel<true, true, 8192> : topk_long_rows_kernel<true, false, 8192>)
                          : (prev ? topk_long_rows_kernel<true, true, 4096> : topk_long_rows_kernel<true, false, 4096>);
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)plan.lds_bytes) != hipSuccess)
            return CHIPMUNK_ERR_LAUNCH;
        hipLaunchKernelGGL(kernel, grid, block_long, plan.lds_bytes, s, cur, prev, C, ld, k, idx, counts, k_stride,
                           plan.seg_cap);
    } else {
        auto kernel = prev ? topk_long_rows_kernel<false, true, 4096> : topk_long_rows_kernel<false, false, 4096>;
        hipLaunchKernelGGL(kernel, grid, block_long, (kBins + kLongSmall) * sizeof(uint32_t), s, cur, prev, C, ld, k, idx,
                           counts, k_stride, 0);
    }
    return launch_status();
}
