// Column-sparse delta attention for gfx950 (Sec. 3.3.1 "Sparse Delta Steps",
// Alg. 3), and dense attention as the special case "every column selected".
//
// One workgroup (4 waves) owns one chunk of c query rows of one (batch, head).
// It walks the chunk's selected key columns in tiles of 64: the K and V rows
// named by the index list are gathered from global memory straight into LDS
// (16-byte asynchronous loads, one K or V row = E*2 contiguous bytes), double
// buffered, and consumed by bf16 MFMA 16x16x32 with an fp32 online softmax.
//
// Register-level layout.  Scores are produced transposed, S^T = K Q^T, so a
// lane holds, for ONE query (lane % 16), the scores of 4 key rows per 16-row
// block (rows 4*(lane/16)+0..3).  Two such blocks are exactly the 8 contraction
// entries the lane must supply as the B operand of O^T += V^T P^T, so the
// probabilities go from the softmax into the second MFMA without leaving
// registers.  V^T tiles come from LDS through the transposing 64-bit read.
// Each wave owns NQB blocks of 16 queries (c = 64*NQB).
#include "common.h"

namespace chipmunk {

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const uint16_t* base;
    uint16_t* out;
    const int32_t* idx;
    const int32_t* counts;
    float* row_m2;  // optional [B,H,N]: reference max used per row, in log2 units
    float* row_l;   // optional [B,H,N]: softmax denominator relative to row_m2
    int N, NB, c, k_stride;
    float sl2;      // softmax_scale * log2(e)
    float o_scale;
};

constexpr int kTileRows = 64;       // key rows per LDS tile
constexpr float kRescaleSlack = 8.f;  // running max may lag the true max by 2^8 before a rescale

// XOR swizzle of the 16-byte chunk position inside a row of the LDS tile,
// chosen so that both the 128-bit K reads (16 rows, one chunk) and the
// transposing V reads (8 rows x 32 bytes) fall on distinct banks.
template <int E>
__device__ __forceinline__ int swizzle(int row) {
    if (E == 128) return ((row & 7) << 1) | ((row >> 3) & 1);
    return (row >> 1) & 7;
}

template <int E, int NQB>
struct AttnState {
    f32x4 O[E / 16][NQB];
    bf16x8 Q[E / 32][NQB];
    float m2[NQB];    // running reference max, in log2 units (score * sl2)
    float lsum[NQB];  // this lane's share of the softmax denominator
};

template <int E, int NQB>
__device__ __forceinline__ void attn_substep(AttnState<E, NQB>& st, const uint8_t* sK, const uint8_t* sV,
                                             int koff, int voff, int kv0, int count, float sl2, int g) {
    constexpr int ROWB = E * 2;
    f32x4 S[2][NQB];
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int qb = 0; qb < NQB; qb++) S[u][qb] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int es = 0; es < E / 32; es++) {
#pragma unroll
        for (int u = 0; u < 2; u++) {
            bf16x8 kop = *reinterpret_cast<const bf16x8*>(sK + u * 16 * ROWB + (koff ^ (64 * es)));
#pragma unroll
            for (int qb = 0; qb < NQB; qb++)
                S[u][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop, st.Q[es][qb], S[u][qb], 0, 0, 0);
        }
    }
    if (kv0 + 32 > count) {  // last, partly filled group of 32 rows: rows at or beyond count do not exist
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                bool dead = kv0 + u * 16 + 4 * g + r >= count;
#pragma unroll
                for (int qb = 0; qb < NQB; qb++)
                    if (dead) S[u][qb][r] = -INFINITY;
            }
    }
    // online softmax over the selected columns; the reference max is raised lazily
    float mx[NQB];
    bool need = false;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float a = fmaxf(fmaxf(S[0][qb][0], S[0][qb][1]), fmaxf(S[0][qb][2], S[0][qb][3]));
        float b = fmaxf(fmaxf(S[1][qb][0], S[1][qb][1]), fmaxf(S[1][qb][2], S[1][qb][3]));
        mx[qb] = rows4_max(fmaxf(a, b)) * sl2;
        need |= mx[qb] > st.m2[qb] + kRescaleSlack;
    }
    if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
        for (int qb = 0; qb < NQB; qb++) {
            float mnew = fmaxf(st.m2[qb], mx[qb]);
            float alpha = __builtin_amdgcn_exp2f(st.m2[qb] - mnew);
            st.m2[qb] = mnew;
            st.lsum[qb] *= alpha;
#pragma unroll
            for (int eb = 0; eb < E / 16; eb++) st.O[eb][qb] *= alpha;
        }
    }
    bf16x8 pop[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float pv[8];
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                pv[u * 4 + r] = __builtin_amdgcn_exp2f(__builtin_fmaf(S[u][qb][r], sl2, -st.m2[qb]));
                st.lsum[qb] += pv[u * 4 + r];
            }
        u32x4 packed;
#pragma unroll
        for (int t = 0; t < 4; t++) packed[t] = pack_bf16x2(pv[2 * t], pv[2 * t + 1]);
        pop[qb] = __builtin_bit_cast(bf16x8, packed);
    }
#pragma unroll
    for (int eb = 0; eb < E / 16; eb++) {
        int a = voff ^ (32 * eb);
        short4v lo = lds_read_tr16(sV + a);
        short4v hi = lds_read_tr16(sV + 16 * ROWB + a);
        typedef __attribute__((ext_vector_type(8))) short short8v;
        short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 vop = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int qb = 0; qb < NQB; qb++)
            st.O[eb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop[qb], st.O[eb][qb], 0, 0, 0);
    }
}

template <int E, int NQB>
__global__ __launch_bounds__(256, 2) void attn_sparse_delta_kernel(AttnParams p) {
    constexpr int ROWB = E * 2;           // bytes per K/V row
    constexpr int CH = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 64 / CH;          // rows covered by one wave-wide 16-byte load
    constexpr int NI = kTileRows / (RPI * 4);  // such loads per wave per tile
    constexpr int TILE = kTileRows * ROWB;

    // two stages, each a K tile followed by a V tile
    __shared__ __attribute__((aligned(1024))) uint8_t smem[4 * TILE];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int g = lane >> 4;
    const int l16 = lane & 15;

    const int64_t unit = blockIdx.x;
    const int64_t bh = unit / p.NB;
    const int chunk = (int)(unit % p.NB);
    const int row0 = chunk * p.c;
    const int rows_valid = min(p.c, p.N - row0);
    const int count = p.counts ? p.counts[unit] : p.N;
    const int32_t* idxp = p.idx ? p.idx + unit * (int64_t)p.k_stride : nullptr;

    const int64_t head_off = bh * (int64_t)p.N * E;
    const uint16_t* qh = p.q + head_off;
    const uint16_t* kh = p.k + head_off;
    const uint16_t* vh = p.v + head_off;
    const uint16_t* baseh = p.base ? p.base + head_off : nullptr;
    uint16_t* outh = p.out + head_off;

    if (count <= 0) {  // nothing selected: the output is the cache, bit for bit
        for (int t = tid; t < rows_valid * CH; t += 256) {
            int64_t off = (int64_t)(row0 + t / CH) * E + (t % CH) * 8;
            u32x4 val = baseh ? *reinterpret_cast<const u32x4*>(baseh + off) : u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(outh + off) = val;
        }
        return;
    }

    AttnState<E, NQB> st;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        st.m2[qb] = -INFINITY;
        st.lsum[qb] = 0.f;
#pragma unroll
        for (int eb = 0; eb < E / 16; eb++) st.O[eb][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        int qrow = (w * NQB + qb) * 16 + l16;
#pragma unroll
        for (int es = 0; es < E / 32; es++) {
            u32x4 val = u32x4{0, 0, 0, 0};
            if (qrow < rows_valid)
                val = *reinterpret_cast<const u32x4*>(qh + (int64_t)(row0 + qrow) * E + 32 * es + 8 * g);
            st.Q[es][qb] = __builtin_bit_cast(bf16x8, val);
        }
    }
    const bool wave_active = w * NQB * 16 < rows_valid;

    // per-lane LDS read offsets (bytes) inside a 16-row group of a tile
    const int koff = l16 * ROWB + ((g ^ swizzle<E>(l16)) * 16);
    const int vrow = 4 * g + (l16 >> 2);
    const int voff = vrow * ROWB + (((((l16 & 3) >> 1)) ^ swizzle<E>(vrow)) * 16) + 8 * (l16 & 1);

    // Gather bookkeeping.  Load i of this wave fills rows (i*4+w)*RPI + lane/CH of
    // the tile; the lane owns LDS chunk position lane%CH of its row and therefore
    // fetches the logical chunk  position ^ swizzle(row).
    const int grow0 = w * RPI + lane / CH;  // row of load 0; load i adds 4*RPI*i
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (uint32_t)w * 1024u);
    const int ntiles = (count + kTileRows - 1) / kTileRows;

    // Selected column per load, fetched one tile ahead and not touched until the
    // gather that uses it (so the index fetch never stalls behind the transfers).
    int cols[NI];
    auto load_cols = [&](int t) {
#pragma unroll
        for (int i = 0; i < NI; i++) {
            int pos = min(t * kTileRows + grow0 + 4 * RPI * i, count - 1);
            cols[i] = idxp ? idxp[pos] : pos;
        }
    };
    auto gather = [&](int stage) {
#pragma unroll
        for (int i = 0; i < NI; i++) {
            int row = grow0 + 4 * RPI * i;
            // byte offset of this lane's chunk inside the head's K (and V) matrix
            uint32_t goff = (uint32_t)cols[i] * ROWB + (uint32_t)(((lane % CH) ^ swizzle<E>(row)) * 16);
            uint32_t dst = lds0 + (uint32_t)(stage * 2 * TILE + i * 4096);
            load_global_to_lds_16B(kh, goff, dst);
            load_global_to_lds_16B(vh, goff, dst + TILE);
        }
    };

    load_cols(0);
    gather(0);
    if (ntiles > 1) load_cols(1);

    for (int t = 0; t < ntiles; t++) {
        const int stage = t & 1;
        wait_all_memory();
        __syncthreads();  // tile t has landed in its stage; every wave is done with the other stage
        if (t + 1 < ntiles) {
            gather(stage ^ 1);
            if (t + 2 < ntiles) load_cols(t + 2);
        }
        if (wave_active) {
            const uint8_t* cK = smem + stage * 2 * TILE;
            const uint8_t* cV = cK + TILE;
            const int kv0 = t * kTileRows;
            attn_substep<E, NQB>(st, cK, cV, koff, voff, kv0, count, p.sl2, g);
            if (kv0 + 32 < count)
                attn_substep<E, NQB>(st, cK + 32 * ROWB, cV + 32 * ROWB, koff, voff, kv0 + 32, count, p.sl2, g);
        }
    }

    if (!wave_active) return;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float ltot = rows4_sum(st.lsum[qb]);
        float f = p.o_scale / ltot;
        int qrow = (w * NQB + qb) * 16 + l16;
        if (qrow < rows_valid) {
            if (p.row_m2 && g == 0) {
                p.row_m2[bh * p.N + row0 + qrow] = st.m2[qb];
                p.row_l[bh * p.N + row0 + qrow] = ltot;
            }
#pragma unroll
            for (int eb = 0; eb < E / 16; eb++) {
                int64_t off = (int64_t)(row0 + qrow) * E + eb * 16 + 4 * g;
                u32x2 b = baseh ? *reinterpret_cast<const u32x2*>(baseh + off) : u32x2{0, 0};
                float o0 = bf16_bits_to_float(b[0] & 0xffffu) + f * st.O[eb][qb][0];
                float o1 = bf16_bits_to_float(b[0] >> 16) + f * st.O[eb][qb][1];
                float o2 = bf16_bits_to_float(b[1] & 0xffffu) + f * st.O[eb][qb][2];
                float o3 = bf16_bits_to_float(b[1] >> 16) + f * st.O[eb][qb][3];
                u32x2 r2 = {pack_bf16x2(o0, o1), pack_bf16x2(o2, o3)};
                *reinterpret_cast<u32x2*>(outh + off) = r2;
            }
        }
    }
}

// Exact column sums of the attention probabilities (Sec. 3.3.1, the tensor D):
//   D[b,h,i,j] = sum over the rows q of chunk i of exp2(s_qj*sl2 - m2_q) / l_q
// with (m2_q, l_q) from the dense attention pass.  Scores are produced as
// S = Q K^T (queries on the rows of the MFMA result), so that the sum over the
// chunk's queries is a sum over a lane's registers, the wave's four 16-lane
// rows and the workgroup's four waves.
struct ColsumParams {
    const uint16_t* q;
    const uint16_t* k;
    const float* row_m2;
    const float* row_l;
    float* colsum;
    int64_t ld;
    int N, NB, c;
    float sl2;
};

template <int E, int NQB>
__global__ __launch_bounds__(256, 2) void attn_colsum_kernel(ColsumParams p) {
    constexpr int ROWB = E * 2;
    constexpr int CH = ROWB / 16;
    constexpr int RPI = 64 / CH;
    constexpr int NI = kTileRows / (RPI * 4);
    constexpr int TILE = kTileRows * ROWB;
    __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * TILE];
    __shared__ float s_part[2][4][kTileRows];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = lane >> 4, l16 = lane & 15;
    const int64_t unit = blockIdx.x;
    const int64_t bh = unit / p.NB;
    const int chunk = (int)(unit % p.NB);
    const int row0 = chunk * p.c;
    const int rows_valid = min(p.c, p.N - row0);
    const uint16_t* qh = p.q + bh * (int64_t)p.N * E;
    const uint16_t* kh = p.k + bh * (int64_t)p.N * E;
    float* drow = p.colsum + unit * p.ld;

    bf16x8 Q[E / 32][NQB];
    float m2v[NQB][4], il[NQB][4];
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        int qrow = (w * NQB + qb) * 16 + l16;
#pragma unroll
        for (int es = 0; es < E / 32; es++) {
            u32x4 val = u32x4{0, 0, 0, 0};
            if (qrow < rows_valid)
                val = *reinterpret_cast<const u32x4*>(qh + (int64_t)(row0 + qrow) * E + 32 * es + 8 * g);
            Q[es][qb] = __builtin_bit_cast(bf16x8, val);
        }
#pragma unroll
        for (int r = 0; r < 4; r++) {  // the MFMA result holds query 4g+r of the block in register r
            int qr = (w * NQB + qb) * 16 + 4 * g + r;
            bool ok = qr < rows_valid;
            m2v[qb][r] = ok ? p.row_m2[bh * p.N + row0 + qr] : 0.f;
            il[qb][r] = ok ? 1.f / p.row_l[bh * p.N + row0 + qr] : 0.f;
        }
    }
    const int koff = l16 * ROWB + ((g ^ swizzle<E>(l16)) * 16);
    const int grow0 = w * RPI + lane / CH;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (uint32_t)w * 1024u);
    const int ntiles = (p.N + kTileRows - 1) / kTileRows;

    auto gather = [&](int t, int stage) {
#pragma unroll
        for (int i = 0; i < NI; i++) {
            int row = grow0 + 4 * RPI * i;
            int pos = min(t * kTileRows + row, p.N - 1);
            uint32_t goff = (uint32_t)pos * ROWB + (uint32_t)(((lane % CH) ^ swizzle<E>(row)) * 16);
            load_global_to_lds_16B(kh, goff, lds0 + (uint32_t)(stage * TILE + i * 4096));
        }
    };
    auto flush = [&](int t) {  // sums of tile t: four waves' partials -> global
        if (tid < kTileRows) {
            int j = t * kTileRows + tid;
            float v = s_part[t & 1][0][tid] + s_part[t & 1][1][tid] + s_part[t & 1][2][tid] + s_part[t & 1][3][tid];
            if (j < p.N) drow[j] = v;
        }
    };

    gather(0, 0);
    for (int t = 0; t < ntiles; t++) {
        const int stage = t & 1;
        wait_all_memory();
        __syncthreads();
        if (t + 1 < ntiles) gather(t + 1, stage ^ 1);
        if (t > 0) flush(t - 1);
        const uint8_t* cK = smem + stage * TILE;
#pragma unroll
        for (int sub = 0; sub < 2; sub++) {
            f32x4 S[2][NQB];
#pragma unroll
            for (int u = 0; u < 2; u++)
#pragma unroll
                for (int qb = 0; qb < NQB; qb++) S[u][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int es = 0; es < E / 32; es++)
#pragma unroll
                for (int u = 0; u < 2; u++) {
                    bf16x8 kop = *reinterpret_cast<const bf16x8*>(cK + (sub * 32 + u * 16) * ROWB + (koff ^ (64 * es)));
#pragma unroll
                    for (int qb = 0; qb < NQB; qb++)
                        S[u][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(Q[es][qb], kop, S[u][qb], 0, 0, 0);
                }
#pragma unroll
            for (int u = 0; u < 2; u++) {
                float part = 0.f;
#pragma unroll
                for (int qb = 0; qb < NQB; qb++)
#pragma unroll
                    for (int r = 0; r < 4; r++)
                        part += __builtin_amdgcn_exp2f(__builtin_fmaf(S[u][qb][r], p.sl2, -m2v[qb][r])) * il[qb][r];
                part = rows4_sum(part);
                if (g == 0) s_part[t & 1][w][sub * 32 + u * 16 + l16] = part;
            }
        }
    }
    __syncthreads();
    flush(ntiles - 1);
}

static int32_t launch_attn(const AttnParams& p, int E, int64_t units, hipStream_t s) {
    dim3 grid((unsigned)units), block(256);
    if (E == 128 && p.c == 192)
        hipLaunchKernelGGL((attn_sparse_delta_kernel<128, 3>), grid, block, 0, s, p);
    else if (E == 128 && p.c == 128)
        hipLaunchKernelGGL((attn_sparse_delta_kernel<128, 2>), grid, block, 0, s, p);
    else if (E == 64 && p.c == 192)
        hipLaunchKernelGGL((attn_sparse_delta_kernel<64, 3>), grid, block, 0, s, p);
    else
        hipLaunchKernelGGL((attn_sparse_delta_kernel<64, 2>), grid, block, 0, s, p);
    return launch_status();
}

}  // namespace chipmunk

using namespace chipmunk;

extern "C" int32_t chipmunk_attn_sparse_delta(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                              const int32_t* idx, const int32_t* counts,
                                              const uint16_t* base, uint16_t* out, int B, int H, int N,
                                              int E, int c, int k_stride, float softmax_scale,
                                              float o_scale, void* stream) {
    if (!q || !k || !v || !out) return CHIPMUNK_ERR_NULL;
    if ((idx == nullptr) != (counts == nullptr)) return CHIPMUNK_ERR_NULL;
    if (idx && !base) return CHIPMUNK_ERR_NULL;
    if (B < 1 || H < 1 || N < 1 || k_stride < 0) return CHIPMUNK_ERR_SHAPE;
    if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY) || !(o_scale == o_scale)) return CHIPMUNK_ERR_SHAPE;
    if (E != 64 && E != 128) return CHIPMUNK_ERR_UNSUPPORTED;
    if (c != 128 && c != 192) return CHIPMUNK_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(base) ||
        !aligned16(idx) || !aligned16(counts))
        return CHIPMUNK_ERR_ALIGN;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    if (units > 0x7fffffffLL) return CHIPMUNK_ERR_SHAPE;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = base; p.out = out; p.idx = idx; p.counts = counts;
    p.row_m2 = nullptr; p.row_l = nullptr;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = k_stride;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = o_scale;
    return launch_attn(p, E, units, (hipStream_t)stream);
}

extern "C" size_t chipmunk_attn_dense_workspace_bytes(int B, int H, int N) {
    if (B < 1 || H < 1 || N < 1) return 0;
    return (size_t)B * H * N * 2 * sizeof(float);
}

extern "C" int32_t chipmunk_attn_dense(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                                       float* colsum, int64_t ld_colsum, int B, int H, int N, int E, int c,
                                       float softmax_scale, void* ws, size_t ws_bytes, void* stream) {
    if (!q || !k || !v || !out) return CHIPMUNK_ERR_NULL;
    if (B < 1 || H < 1 || N < 1) return CHIPMUNK_ERR_SHAPE;
    if (!(softmax_scale > 0.f) || !(softmax_scale < INFINITY)) return CHIPMUNK_ERR_SHAPE;
    if (E != 64 && E != 128) return CHIPMUNK_ERR_UNSUPPORTED;
    if (c != 128 && c != 192) return CHIPMUNK_ERR_UNSUPPORTED;
    if (colsum && ld_colsum < N) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(colsum) || !aligned16(ws) ||
        (colsum && (ld_colsum % 4) != 0))
        return CHIPMUNK_ERR_ALIGN;
    if (colsum && (!ws || ws_bytes < chipmunk_attn_dense_workspace_bytes(B, H, N))) return CHIPMUNK_ERR_WORKSPACE;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    if (units > 0x7fffffffLL) return CHIPMUNK_ERR_SHAPE;
    hipStream_t s = (hipStream_t)stream;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = nullptr; p.out = out; p.idx = nullptr; p.counts = nullptr;
    p.row_m2 = colsum ? (float*)ws : nullptr;
    p.row_l = colsum ? (float*)ws + (int64_t)B * H * N : nullptr;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = 0;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = 1.f;
    int32_t st = launch_attn(p, E, units, s);
    if (st != CHIPMUNK_OK || !colsum) return st;
    ColsumParams cp;
    cp.q = q; cp.k = k; cp.row_m2 = p.row_m2; cp.row_l = p.row_l; cp.colsum = colsum; cp.ld = ld_colsum;
    cp.N = N; cp.NB = NB; cp.c = c; cp.sl2 = p.sl2;
    dim3 grid((unsigned)units), block(256);
    if (E == 128 && c == 192) hipLaunchKernelGGL((attn_colsum_kernel<128, 3>), grid, block, 0, s, cp);
    else if (E == 128 && c == 128) hipLaunchKernelGGL((attn_colsum_kernel<128, 2>), grid, block, 0, s, cp);
    else if (E == 64 && c == 192) hipLaunchKernelGGL((attn_colsum_kernel<64, 3>), grid, block, 0, s, cp);
    else hipLaunchKernelGGL((attn_colsum_kernel<64, 2>), grid, block, 0, s, cp);
    return launch_status();
}
