// Column-sparse delta attention for gfx950 (Sec. 3.3.1 "Sparse Delta Steps",
// Alg. 3), and dense attention as the special case "every column selected".
//
// One workgroup (4 waves) owns one chunk of c query rows of one (batch, head).
// It walks the chunk's selected key columns in tiles of 32: the K and V rows
// named by the index list are gathered from global memory straight into LDS
// (16-byte asynchronous loads, one K or V row = E*2 contiguous bytes), two
// tiles per workgroup barrier and double buffered: the two tiles of the next
// step are in flight while the two of this step are consumed by bf16 MFMA
// 16x16x32 with an fp32 online softmax.  Two workgroups share a compute unit
// (two waves per SIMD): a wave hides nothing behind its own MFMAs, the other
// wave's vector and LDS instructions are what runs in their shadow.
//
// Register-level layout.  Scores are produced transposed, S^T = K Q^T, so a
// lane holds, for ONE query (lane % 16), the scores of 4 key rows per 16-row
// block (rows 4*(lane/16)+0..3).  Two such blocks are exactly the 8 contraction
// entries the lane must supply as the B operand of O^T += V^T P^T, so the
// probabilities go from the softmax into the second MFMA without leaving
// registers.  V^T tiles come from LDS through the transposing 64-bit read.
// Each wave owns NQB blocks of 16 queries (c = 64*NQB).
#include "common.h"

#include <type_traits>

namespace chipmunk {

struct AttnParams {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const uint16_t* base;
    uint16_t* out;
    const int32_t* idx;
    const int32_t* counts;
    float* row_m;   // optional [B,H,N]: the reference the row's exponentials were taken against, in units of the
                    // scaled scores (natural logarithm); within 2^8 of the row maximum, not necessarily equal to it
    float* row_l;   // optional [B,H,N]: sum_j exp(score_j - row_m)
    int N, NB, c, k_stride;
    float sl2;      // softmax_scale * log2(e)
    float o_scale;
    // fused column sums with given normalisers (Alg. 4): dense launches of the FUSED kernel only
    const float* prev_m;   // [B,H,N], natural-log units like row_m
    const float* prev_l;   // [B,H,N]
    float* colsum;         // [B,H,NB,ld_colsum]
    int64_t ld_colsum;
};

constexpr int kTileRows = 32;         // key rows per LDS tile = one step of the online softmax
constexpr int kTilesPerStep = 2;      // tiles consumed between two workgroup barriers
constexpr int kStages = 2 * kTilesPerStep;  // tile buffers (K tile + V tile each): one step in use, one in flight
constexpr int kColsumTileRows = 64;   // the column-sum kernel keeps 64-row tiles, double buffered
constexpr float kRescaleSlack = 8.f;  // running max may lag the true max by 2^8 before a rescale

// XOR swizzle of the 16-byte chunk position inside a row of the LDS tile.  For
// 256-byte rows the map (a GF(2)-linear function of the row's low four bits) was
// picked by measurement on gfx950 among all such maps: it is free of bank
// conflicts both for the 128-bit K reads (16 rows, one chunk each per 16 lanes)
// and for the transposing 64-bit V reads (4 rows x 32 bytes per 16 lanes).
template <int E>
__device__ __forceinline__ int swizzle(int row) {
    if (E == 128) return ((row & 1) << 1) ^ (((row >> 1) & 1) * 9) ^ (((row >> 2) & 1) << 2) ^ (((row >> 3) & 1) << 1);
    return (row >> 1) & 7;
}

template <int E, int NQB>
struct AttnState {
    f32x4 O[E / 16][NQB];
    f32x4 L[NQB];     // softmax denominator, accumulated by the MFMA against a row of ones
    bf16x8 Q[E / 32][NQB];
    f32x4 negm[NQB];  // -m in all four registers (m: the running reference max, in units of the raw scores <q,k>; it
                      // is replaced by the first tile's row maximum): the C operand that starts every score accumulation
};

// The work on one tile of 32 selected key rows is split in three pieces so that
// the kernel can software-pipeline them: scores of tile t+1 (MFMA) are issued
// next to the exponentials of tile t (VALU), and the max bookkeeping of tile t+1
// (VALU) next to the P.V products of tile t (MFMA).

// LDS reads take byte addresses in registers (the LDS base is already added) plus compile-time offsets, so that the
// offsets become the immediate field of the read instead of an address computation per read.
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>((uintptr_t)addr);
}
__device__ __forceinline__ short4v lds_read_tr16_at(uint32_t addr) {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<__attribute__((address_space(3))) short4v*>((uintptr_t)addr));
}

// S^T = K Q^T - m for one tile: raw scores relative to the reference max (the MFMA adds -m for free where a
// separate subtraction would cost one vector instruction per score).  kaddr[es]: the lane's read address for
// contraction slice es in tile buffer 0; tile_off: byte offset of the tile buffer (compile-time at the call).
// between(j), j = 0 .. E/16 - 1, is called after the j-th group of NQB products: the kernel issues one of the next
// step's tile transfers there, so that the transfers are spread over the products instead of queueing up in one
// burst during which the wave issues nothing else.
// K operands are requested KPF groups ahead of the products that consume them.  One group ahead is enough: the
// other wave of the SIMD covers what latency is left, and deeper prefetch only costs registers (measured equal
// for the column-sparse launch, 2 % slower for the dense one)
template <int E, int NQB, int KPF, typename Between>
__device__ __forceinline__ void attn_scores(f32x4 (&S)[2][NQB], const AttnState<E, NQB>& st, const uint32_t (&kaddr)[E / 32],
                                            int tile_off, Between&& between) {
    constexpr int ROWB = E * 2;
    constexpr int NG = E / 16;   // groups of NQB products: group j = contraction slice j / 2, key rows 16 (j % 2) ..
    bf16x8 kop[NG];
#pragma unroll
    for (int j = 0; j < KPF; j++) kop[j] = lds_read_b128(kaddr[j / 2] + tile_off + (j % 2) * 16 * ROWB);
    __builtin_amdgcn_sched_group_barrier(0x100, KPF, 0);  // the LDS reads lead the block
#pragma unroll
    for (int j = 0; j < NG; j++) {
        const int es = j / 2, u = j % 2;
        if (j + KPF < NG) {
            const int jn = j + KPF;
            kop[jn] = lds_read_b128(kaddr[jn / 2] + tile_off + (jn % 2) * 16 * ROWB);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int qb = 0; qb < NQB; qb++)
            S[u][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[j], st.Q[es][qb], es == 0 ? st.negm[qb] : S[u][qb], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NQB, 0);
        between(j);
    }
}

// Inside a step (kTilesPerStep tiles) the rows of the LDS tiles are a fixed permutation of the step's list
// positions: every lane of the gather fetches kTilesPerStep * NI consecutive positions (one vector load of column
// numbers) and deals them out over the tiles.  Row q of tile s holds list position  step_base + list_pos(s, q).
// The softmax does not care about the order; only the mask of the unit's last tiles and the column sums do.
template <int E>
__device__ __forceinline__ int list_pos_in_step(int s, int q) {
    constexpr int NI = E / 64;                       // gather loads per wave, tile and matrix
    constexpr int LANEROWS = kTileRows / NI;         // rows of a tile that one such load of every wave covers
    return (q % LANEROWS) * (kTilesPerStep * NI) + s * NI + q / LANEROWS;
}

// The last tiles of a unit: rows whose list position is at or beyond `count` score -inf.
template <int E, int NQB>
__device__ __forceinline__ void attn_mask_tail(f32x4 (&S)[2][NQB], int step_base, int s, int count, int g) {
#pragma unroll
    for (int u = 0; u < 2; u++)
#pragma unroll
        for (int r = 0; r < 4; r++) {
            bool dead = step_base + list_pos_in_step<E>(s, u * 16 + 4 * g + r) >= count;
#pragma unroll
            for (int qb = 0; qb < NQB; qb++)
                if (dead) S[u][qb][r] = -INFINITY;
        }
}

// Raise the reference max where this tile's relative scores exceed the slack
// (2^8 in probability, given here in raw score units); O, the denominator and the
// tile's relative scores are rescaled (rare after the first tiles).  The common
// case costs a lane only the max over its own 8 scores per query block: the reduction over the four lanes that share a query runs when some
// lane of the wave has seen an excess.  The first tile of a unit sets the
// reference to the tile's row maximum, whatever its sign.
template <int E, int NQB>
__device__ __forceinline__ void attn_update_max(AttnState<E, NQB>& st, f32x4 (&S)[2][NQB], bool first, float sl2,
                                                float slack) {
    float mx[NQB];
    bool need = first;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float a = fmaxf(fmaxf(S[0][qb][0], S[0][qb][1]), S[0][qb][2]);
        float b = fmaxf(fmaxf(a, S[0][qb][3]), S[1][qb][0]);
        float c = fmaxf(fmaxf(b, S[1][qb][1]), S[1][qb][2]);
        mx[qb] = fmaxf(c, S[1][qb][3]);
        need |= mx[qb] > slack;
    }
    if (__builtin_amdgcn_ballot_w64(need) != 0) {
#pragma unroll
        for (int qb = 0; qb < NQB; qb++) {
            float d = rows4_max(mx[qb]);             // the tile's row maximum relative to the reference
            float up = first ? d : fmaxf(d, 0.f);    // the reference only rises, except when it is first set
            float alpha = first ? 1.f : __builtin_amdgcn_exp2f(-up * sl2);   // O and L are still zero on the first tile
            const float nm = st.negm[qb][0] - up;
            st.negm[qb] = f32x4{nm, nm, nm, nm};
            st.L[qb] *= alpha;
#pragma unroll
            for (int eb = 0; eb < E / 16; eb++) st.O[eb][qb] *= alpha;
#pragma unroll
            for (int u = 0; u < 2; u++)
#pragma unroll
                for (int r = 0; r < 4; r++) S[u][qb][r] -= up;
        }
    }
}

// P = exp2(S*sl2) in bf16, the denominator, and O^T += V^T P^T.
// The transposing V reads do not depend on the probabilities: the first kVPrefetch
// operands are requested before the exponentials, the rest kVPrefetch steps ahead
// of the MFMAs that consume them, so LDS latency stays off the MFMA chain.
constexpr int kVPrefetch = 2;        // (1 in the kernel with the column sums)

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x) {  // x of the lane that the DPP control CTRL names
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}

// acc[4 u + r] is the lane's value for tile key row 16 u + 4 g + r.  Sums each of the eight over the 16 lanes of
// the row (the wave's 16 queries of a block) and writes them to part[32] in tile key order.  Halving exchange:
// at each step a lane keeps half of its values and hands the other half to a partner that keeps those, so 8 adds
// stand in for 32.  Partners: lane ^ 15, ^ 7, ^ 3, ^ 1; the value a lane ends with is 4 bit3 + 2 bit2 + bit1.
__device__ __forceinline__ void row16_sums_to_lds(const float (&acc)[8], float* part, int g, int l16) {
    const bool b3 = l16 & 8, b2 = l16 & 4, b1 = l16 & 2;
    float x[4], y[2];
#pragma unroll
    for (int i = 0; i < 4; i++) x[i] = (b3 ? acc[i + 4] : acc[i]) + dpp_f32<0x140>(b3 ? acc[i] : acc[i + 4]);  // row_mirror
#pragma unroll
    for (int i = 0; i < 2; i++) y[i] = (b2 ? x[i + 2] : x[i]) + dpp_f32<0x141>(b2 ? x[i] : x[i + 2]);          // row_half_mirror
    float z = (b1 ? y[1] : y[0]) + dpp_f32<0x1b>(b1 ? y[0] : y[1]);                                              // quad_perm 3,2,1,0
    z += dpp_f32<0xb1>(z);                                                                                       // quad_perm 1,0,3,2
    if (!(l16 & 1)) part[(l16 & 8 ? 16 : 0) + 4 * g + ((l16 >> 1) & 3)] = z;
}

// COLSUM (Alg. 4): also the tile's column sums with given normalisers.  The weight of (key, query) there is
// exp2(score * sl2 - prev_m2) / prev_l = p * wq, with p the probability formed here against the running
// reference st.m and wq = exp2(st.m * sl2 + off) per query, off = -prev_m2 - log2(prev_l) (-inf: no such query).
template <int E, int NQB, bool COLSUM = false, int VPF = kVPrefetch>
__device__ __forceinline__ void attn_weights_and_pv(AttnState<E, NQB>& st, const f32x4 (&S)[2][NQB],
                                                    const uint32_t (&vaddr)[E / 16], int tile_off, float sl2, bf16x8 ones,
                                                    const float* off = nullptr, float* part = nullptr, int g = 0,
                                                    int l16 = 0) {
    constexpr int ROWB = E * 2;
    constexpr int NEB = E / 16;
    typedef __attribute__((ext_vector_type(8))) short short8v;
    short4v vlo[NEB], vhi[NEB];
#pragma unroll
    for (int eb = 0; eb < VPF; eb++) {
        vlo[eb] = lds_read_tr16_at(vaddr[eb] + tile_off);
        vhi[eb] = lds_read_tr16_at(vaddr[eb] + tile_off + 16 * ROWB);
    }
    __builtin_amdgcn_sched_group_barrier(0x100, 2 * VPF, 0);  // the LDS reads lead the block
    bf16x8 pop[NQB];
    float acc[8];
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float pv[8];
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
            for (int r = 0; r < 4; r++)
                pv[u * 4 + r] = __builtin_amdgcn_exp2f(S[u][qb][r] * sl2);
        if (COLSUM) {
            // the cap keeps wq finite, so that a zero probability times it stays zero
            const float wq = __builtin_amdgcn_exp2f(fminf(__builtin_fmaf(-st.negm[qb][0], sl2, off[qb]), 126.f));
#pragma unroll
            for (int j = 0; j < 8; j++) acc[j] = qb == 0 ? pv[j] * wq : __builtin_fmaf(pv[j], wq, acc[j]);
        }
        u32x4 packed;
#pragma unroll
        for (int t = 0; t < 4; t++) packed[t] = pack_bf16x2(pv[2 * t], pv[2 * t + 1]);
        pop[qb] = __builtin_bit_cast(bf16x8, packed);
    }
    if (COLSUM) row16_sums_to_lds(acc, part, g, l16);
    // denominator from the same bf16 probabilities that weight V
#pragma unroll
    for (int qb = 0; qb < NQB; qb++)
        st.L[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pop[qb], st.L[qb], 0, 0, 0);
    __builtin_amdgcn_sched_group_barrier(0x008, NQB, 0);
#pragma unroll
    for (int eb = 0; eb < NEB; eb++) {
        if (eb + VPF < NEB) {
            vlo[eb + VPF] = lds_read_tr16_at(vaddr[eb + VPF] + tile_off);
            vhi[eb + VPF] = lds_read_tr16_at(vaddr[eb + VPF] + tile_off + 16 * ROWB);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        short8v both = __builtin_shufflevector(vlo[eb], vhi[eb], 0, 1, 2, 3, 4, 5, 6, 7);
        bf16x8 vop = __builtin_bit_cast(bf16x8, both);
#pragma unroll
        for (int qb = 0; qb < NQB; qb++)
            st.O[eb][qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop, pop[qb], st.O[eb][qb], 0, 0, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, NQB, 0);
    }
}

constexpr int kBlockColumns = CHIPMUNK_ATTN_BLOCK_COLUMNS;   // key columns per entry of a block list
static_assert(kBlockColumns % (kTilesPerStep * kTileRows) == 0, "a step never straddles two blocks");

// What the kernel walks.  kColumnList: the unit's list of columns.  kEveryColumn: no list, every column (dense).
// kFusedDense: every column, and the column sums of Alg. 4 are formed from the same score tiles.  kBlockList: the
// unit's list names blocks of kBlockColumns consecutive columns (the [c, 128] block sparsity of Table 2); the list
// positions are the blocks' columns in order, so the rows of a step are one contiguous run of K and V.
enum AttnMode { kColumnList = 0, kFusedDense = 1, kBlockList = 2, kEveryColumn = 3 };

// NWAVES waves per workgroup, each owning NQB blocks of 16 queries: c = 16 * NQB * NWAVES.
template <int E, int NQB, int NWAVES, int MODE = kColumnList>
__global__ __launch_bounds__(64 * NWAVES, NWAVES == 4 ? 2 : 1) void attn_sparse_delta_kernel(AttnParams p) {
    constexpr bool FUSED = MODE == kFusedDense;
    constexpr bool BLOCKS = MODE == kBlockList;
    // Every column in order: the columns are the list positions.  A mode of its own and not a null list inside
    // kColumnList: there the branch on the pointer put a wait for all memory behind each step's tile requests (the
    // compiler guards the registers that the other branch loads the column numbers into).
    constexpr bool NOLIST = FUSED || MODE == kEveryColumn;
    constexpr int ROWB = E * 2;           // bytes per K/V row
    constexpr int CH = ROWB / 16;         // 16-byte chunks per row
    constexpr int RPI = 64 / CH;          // rows covered by one wave-wide 16-byte load
    constexpr int NI = kTileRows / (RPI * NWAVES);  // such loads per wave per tile and matrix
    constexpr int NT = 64 * NWAVES;
    constexpr int TILE = kTileRows * ROWB;
    constexpr int STAGE = 2 * TILE;       // K tile then V tile

    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];  // kStages * STAGE bytes
    // FUSED: per-wave column sums of the two tiles of a step, double buffered over steps
    __shared__ float s_part[FUSED ? 2 * NWAVES * kTilesPerStep * kTileRows : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = tid >> 6;
    const int wu = __builtin_amdgcn_readfirstlane(w);
    const int g = lane >> 4;
    const int l16 = lane & 15;

    const int64_t unit = blockIdx.x;
    const int64_t bh = unit / p.NB;
    const int chunk = (int)(unit % p.NB);
    const int row0 = chunk * p.c;
    const int rows_valid = min(p.c, p.N - row0);
    // Contents of counts and idx are the caller's precondition; they are clamped all the same so that a bad
    // entry reads a wrong row instead of leaving the tensors.
    // (block lists: counts and k_stride are in blocks; `count` is in list positions = columns all the same)
    const int entries = __builtin_amdgcn_readfirstlane(p.counts ? min(p.counts[unit], p.k_stride) : p.N);
    int count = BLOCKS ? entries * kBlockColumns : entries;
    // The length is hidden from the compiler's value tracking: knowing that a block list's length is a multiple
    // of two steps, it fuses the two copies of the step below into one scheduling region and then needs far
    // more registers than there are (hundreds of bytes of spills in the main loop).
    asm volatile("" : "+s"(count));

    const int64_t head_off = bh * (int64_t)p.N * E;
    const uint16_t* qh = p.q + head_off;
    const uint16_t* kh = p.k + head_off;
    const uint16_t* vh = p.v + head_off;
    const uint16_t* baseh = p.base ? p.base + head_off : nullptr;
    uint16_t* outh = p.out + head_off;

    if (count <= 0) {  // nothing selected: the output is the cache, bit for bit
        for (int t = tid; t < rows_valid * CH; t += NT) {
            int64_t off = (int64_t)(row0 + t / CH) * E + (t % CH) * 8;
            u32x4 val = baseh ? *reinterpret_cast<const u32x4*>(baseh + off) : u32x4{0, 0, 0, 0};
            *reinterpret_cast<u32x4*>(outh + off) = val;
        }
        return;
    }

    AttnState<E, NQB> st;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        st.negm[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
        st.L[qb] = f32x4{0.f, 0.f, 0.f, 0.f};
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
    const bool wave_active = wu * NQB * 16 < rows_valid;   // wave-uniform, and known to be
    const float slack = kRescaleSlack / p.sl2;
    // FUSED: -prev_m (log2 units) - log2(prev_l) of the lane's queries; -inf drops a query row that does not exist
    float off[NQB];
    if (FUSED) {
#pragma unroll
        for (int qb = 0; qb < NQB; qb++) {
            int qrow = (w * NQB + qb) * 16 + l16;
            off[qb] = -INFINITY;
            if (qrow < rows_valid) {
                const int64_t at = bh * p.N + row0 + qrow;
                off[qb] = -p.prev_m[at] * 1.4426950408889634f - __builtin_amdgcn_logf(p.prev_l[at]);
            }
        }
    }
    const int active_waves = min(NWAVES, (rows_valid + NQB * 16 - 1) / (NQB * 16));
    float* colsum_row = FUSED ? p.colsum + unit * p.ld_colsum : nullptr;
    auto flush_column_sums = [&](int tile0) {  // sums of tiles tile0, tile0+1: the waves' partial sums -> global
        if (FUSED && tid < kTilesPerStep * kTileRows) {
            const float* part = s_part + ((tile0 / kTilesPerStep) & 1) * (NWAVES * kTilesPerStep * kTileRows);
            float v = 0.f;
            for (int ww = 0; ww < active_waves; ww++) v += part[ww * (kTilesPerStep * kTileRows) + tid];
            const int j = tile0 * kTileRows + list_pos_in_step<E>(tid / kTileRows, tid % kTileRows);
            if (j < p.N) colsum_row[j] = v;
        }
    };
    const u32x4 ones_bits = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);

    // per-lane LDS read addresses (bytes, the LDS base included) inside a 16-row group of tile buffer 0: one per
    // contraction slice, because the slice number enters through the XOR swizzle, not additively
    const int koff = l16 * ROWB + ((g ^ swizzle<E>(l16)) * 16);
    const int vrow = 4 * g + (l16 >> 2);
    const int voff = vrow * ROWB + (((((l16 & 3) >> 1)) ^ swizzle<E>(vrow)) * 16) + 8 * (l16 & 1);
    const uint32_t smem_at = (uint32_t)(uintptr_t)CHIPMUNK_LDS_PTR(smem);
    uint32_t kaddr[E / 32], vaddr[E / 16];
#pragma unroll
    for (int es = 0; es < E / 32; es++) kaddr[es] = smem_at + (uint32_t)(koff ^ (64 * es));
#pragma unroll
    for (int eb = 0; eb < E / 16; eb++) vaddr[eb] = smem_at + (uint32_t)(voff ^ (32 * eb));
    // The LDS base is a link-time constant; left visible, the compiler would keep the offsets without it and add
    // it again at every read.  Behind this barrier each address is just a register.
#pragma unroll
    for (int es = 0; es < E / 32; es++) asm volatile("" : "+v"(kaddr[es]));
#pragma unroll
    for (int eb = 0; eb < E / 16; eb++) asm volatile("" : "+v"(vaddr[eb]));

    // Gather bookkeeping.  Load i of this wave fills rows (i*NWAVES+w)*RPI .. +RPI-1 of
    // the tile; the lane owns row (i*NWAVES+w)*RPI + lane/CH, LDS chunk position lane%CH,
    // and therefore fetches the logical chunk  position ^ swizzle(row).
    const int sel = lane / CH;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (uint32_t)w * 1024u);
    // whole steps: the rows of a step's tiles interleave the step's list positions (list_pos_in_step), so the last
    // step runs all its tiles, masked
    const int ntiles = (count + kTilesPerStep * kTileRows - 1) / (kTilesPerStep * kTileRows) * kTilesPerStep;
    uint32_t chunk_off[NI];  // byte offset of the lane's chunk inside the row it fetches
#pragma unroll
    for (int i = 0; i < NI; i++) chunk_off[i] = (uint32_t)(((lane % CH) ^ swizzle<E>((i * NWAVES + w) * RPI + sel)) * 16);

    // K, V and the unit's index list are read through buffer resources: the hardware checks every
    // offset against the tensor's size (an out-of-range access returns zero), so neither the column
    // numbers nor the positions in the list are clamped with vector instructions.  A slot of the list
    // at or beyond `count` reads as column 0: a valid row, whose scores the last tile masks.
    const i32x4 kbuf = raw_buffer_words(kh, (uint32_t)p.N * ROWB);
    const i32x4 vbuf = raw_buffer_words(vh, (uint32_t)p.N * ROWB);
    const int32_t* idxg = !NOLIST && p.idx ? p.idx + unit * (int64_t)p.k_stride : nullptr;
    // two views of the unit's list: its whole row (positions below k_stride: the vector loads of the steps that lie
    // inside the list) and the part below count (a position at or beyond count reads as 0: the list's last step)
    const __amdgpu_buffer_rsrc_t ibuf_row = raw_buffer(idxg, idxg ? (uint32_t)p.k_stride * 4u : 0u);
    const __amdgpu_buffer_rsrc_t ibuf = raw_buffer(idxg, idxg ? (uint32_t)entries * 4u : 0u);

    // Every lane fetches the column numbers of the tile rows it fills, one step ahead of the gather that uses
    // them: the load is issued behind that step's tile transfers and has landed, like those, when the next step
    // starts with its wait for all memory.  A lane's kTilesPerStep * NI rows of a step hold consecutive list
    // positions (list_pos_in_step), so one vector load brings them all.  The list's last step is the only one
    // that can reach beyond count: its columns are fetched once, up front, entry by entry through the view that
    // ends at count (colt), and the step before it (or the prologue) gathers from those.
    constexpr int RPL = kTilesPerStep * NI;       // rows (= column numbers) per lane and step
    static_assert(RPL == 4 || RPL == 2, "the column numbers of a step come as one 16- or 8-byte load per lane");
    int colv[RPL], colt[RPL];
    int next_pos = (w * RPI + sel) * RPL;         // the lane's first list position in the next step to load
    if constexpr (MODE == kColumnList) {
        const int last_pos = (ntiles / kTilesPerStep - 1) * (kTilesPerStep * kTileRows) + next_pos;
#pragma unroll
        for (int j = 0; j < RPL; j++) colt[j] = __builtin_amdgcn_raw_buffer_load_b32(ibuf, (last_pos + j) * 4, 0, 0);
    }
    int blockv = 0;                               // BLOCKS: the block that holds the next step to gather (the same in every lane)
    int block_now = 0, block_next = 0;            // BLOCKS: first column of the block of the step in work / of the next step
    auto load_cols = [&]() {
        if constexpr (NOLIST) return;  // gather_offsets forms the columns from the positions
        if constexpr (BLOCKS) {        // one list entry serves kBlockColumns positions; past the list's end it reads as block 0
            blockv = __builtin_amdgcn_raw_buffer_load_b32(ibuf, (next_pos / kBlockColumns) * 4, 0, 0);
            next_pos += kTilesPerStep * kTileRows;
            return;
        }
        if constexpr (RPL == 4) {
            const u32x4 c4 = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ibuf_row, next_pos * 4, 0, 0));
#pragma unroll
            for (int j = 0; j < RPL; j++) colv[j] = (int)c4[j];
        } else {
            const u32x2 c2 = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(ibuf_row, next_pos * 4, 0, 0));
#pragma unroll
            for (int j = 0; j < RPL; j++) colv[j] = (int)c2[j];
        }
        next_pos += kTilesPerStep * kTileRows;
    };
    // One of the E/16 transfers that fill buffer half `half` with the tiles whose columns are in colv: piece j is
    // the K (j even) or V (j odd) part of load i = (j/2) % NI of tile s = j / (2 NI).
    uint32_t goff[kTilesPerStep][NI];   // byte offset of the lane's chunk inside the head's K (and V) matrix
    // from the column numbers that have landed: once per step, ahead of the products; `last`: the step to gather
    // is the list's last one
    int gather_pos = (w * RPI + sel) * RPL;       // FUSED: the lane's first list position in the next step to gather
    auto gather_offsets = [&](bool last) {
#pragma unroll
        for (int s = 0; s < kTilesPerStep; s++)
#pragma unroll
            for (int i = 0; i < NI; i++) {
                int col;
                if constexpr (NOLIST) col = min(gather_pos + s * NI + i, p.N - 1);   // column = position
                else if constexpr (BLOCKS) col = min(blockv * kBlockColumns + (gather_pos % kBlockColumns) + s * NI + i, p.N - 1);
                else col = last ? colt[s * NI + i] : colv[s * NI + i];
                goff[s][i] = (uint32_t)col * ROWB + chunk_off[i];
                // formed here, not again in front of every transfer (the kernel with the column sums has no
                // registers for that and lets the compiler form them where it likes)
                if constexpr (!FUSED) asm volatile("" : "+v"(goff[s][i]));
            }
        gather_pos += kTilesPerStep * kTileRows;
        if constexpr (BLOCKS) {
            block_now = block_next;
            block_next = __builtin_amdgcn_readfirstlane(blockv) * kBlockColumns;
        }
    };
    auto gather_piece = [&](auto half_c, int j) {
        constexpr int half = decltype(half_c)::value;
        const int s = j / (2 * NI), i = (j / 2) % NI;
        const uint32_t dst = lds0 + (uint32_t)((half * kTilesPerStep + s) * STAGE + i * NWAVES * 1024);
        if (j & 1) load_buffer_to_lds_16B(vbuf, goff[s][i], dst + TILE);
        else load_buffer_to_lds_16B(kbuf, goff[s][i], dst);
    };
    static_assert(kTilesPerStep * NI * 2 == E / 16, "one transfer per group of score products");

    // The query loads must not be left pending into the loop: a wait for them inside
    // the loop would also wait for every tile transfer in flight.  The columns of the
    // first step are requested beside them: one round trip for both.
    load_cols();
    wait_all_memory();

    // first step in flight; columns of the second step requested
    gather_offsets(ntiles <= kTilesPerStep);
#pragma unroll
    for (int j = 0; j < E / 16; j++) gather_piece(std::integral_constant<int, 0>{}, j);
    load_cols();

    // One step: the kTilesPerStep tiles in buffer half `half`.  The half is a compile-time constant (the loop
    // below alternates two copies of the step), so every LDS offset of the step is an immediate of its read.
    // The next step's tiles are requested between the score products of this step's first tile, and the columns
    // of the step after that behind them.  Both happen on every step: past the end of the list the columns read
    // as 0 (the buffer's range check), so the last step fetches row 0 into buffers nobody reads.
    auto step = [&](auto half_c, int t) {
        constexpr int half = decltype(half_c)::value;
        wait_all_memory();
        __syncthreads();  // this step's tiles have landed for every wave; the other half is free to refill
        gather_offsets(t + 2 * kTilesPerStep >= ntiles);
        if (FUSED && t > 0) flush_column_sums(t - kTilesPerStep);
#pragma unroll
        for (int s = 0; s < kTilesPerStep; s++) {
            const int tile_off = (half * kTilesPerStep + s) * STAGE;   // a constant once the loop over s is unrolled
            f32x4 S[2][NQB];
            if (s == 0) {
                attn_scores<E, NQB, 1>(S, st, kaddr, tile_off,
                                    [&](int j) { gather_piece(std::integral_constant<int, half ^ 1>{}, j); });
                load_cols();
            } else {
                attn_scores<E, NQB, 1>(S, st, kaddr, tile_off, [](int) {});
            }
            if constexpr (BLOCKS) {   // only the sequence's last block can reach beyond N; it may stand anywhere in the list
                const int col0 = block_now + (t * kTileRows) % kBlockColumns;
                if (col0 + kTilesPerStep * kTileRows > p.N) attn_mask_tail<E, NQB>(S, col0, s, p.N, g);
            } else {
                if (t + kTilesPerStep >= ntiles) attn_mask_tail<E, NQB>(S, t * kTileRows, s, count, g);
            }
            attn_update_max<E, NQB>(st, S, t + s == 0, p.sl2, slack);
            attn_weights_and_pv<E, NQB, FUSED, FUSED ? 1 : kVPrefetch>(st, S, vaddr, tile_off + TILE, p.sl2, ones, off,
                                               s_part + ((half * NWAVES + w) * kTilesPerStep + s) * kTileRows, g, l16);
        }
    };
#pragma unroll 1
    for (int t = 0; t < ntiles; t += 2 * kTilesPerStep) {
        step(std::integral_constant<int, 0>{}, t);
        if (t + kTilesPerStep >= ntiles) break;
        step(std::integral_constant<int, 1>{}, t + kTilesPerStep);
    }
    // The base rows that the results are merged with are requested here, for every query block at once and in front
    // of the wait for the last step's transfers: one round trip for all of it.  Without a branch: a query row that
    // does not exist reads the chunk's last row, a call without base reads the output buffer; neither value is used.
    const uint16_t* base_src = baseh ? baseh : outh;
    u32x2 bv[NQB][E / 16];
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        int qrow = (w * NQB + qb) * 16 + l16;
        const int64_t row_off = (int64_t)(row0 + min(qrow, rows_valid - 1)) * E + 4 * g;
#pragma unroll
        for (int eb = 0; eb < E / 16; eb++) bv[qb][eb] = *reinterpret_cast<const u32x2*>(base_src + row_off + eb * 16);
    }
    wait_all_memory();  // the last step's transfers into the unused half must have landed before the wave may end
    if (FUSED) {
        __syncthreads();  // the last step's partial sums are complete
        flush_column_sums(((ntiles - 1) / kTilesPerStep) * kTilesPerStep);
    }

    if (!wave_active) return;
#pragma unroll
    for (int qb = 0; qb < NQB; qb++) {
        float ltot = st.L[qb][0];
        float f = p.o_scale / ltot;
        int qrow = (w * NQB + qb) * 16 + l16;
        const int64_t row_off = (int64_t)(row0 + min(qrow, rows_valid - 1)) * E + 4 * g;
        if (qrow < rows_valid) {
            if (p.row_m && g == 0) {
                p.row_m[bh * p.N + row0 + qrow] = -st.negm[qb][0] * (p.sl2 * 0.6931471805599453f);
                p.row_l[bh * p.N + row0 + qrow] = ltot;
            }
#pragma unroll
            for (int eb = 0; eb < E / 16; eb++) {
                u32x2 b = baseh ? bv[qb][eb] : u32x2{0, 0};
                float o0 = bf16_bits_to_float(b[0] & 0xffffu) + f * st.O[eb][qb][0];
                float o1 = bf16_bits_to_float(b[0] >> 16) + f * st.O[eb][qb][1];
                float o2 = bf16_bits_to_float(b[1] & 0xffffu) + f * st.O[eb][qb][2];
                float o3 = bf16_bits_to_float(b[1] >> 16) + f * st.O[eb][qb][3];
                u32x2 r2 = {pack_bf16x2(o0, o1), pack_bf16x2(o2, o3)};
                *reinterpret_cast<u32x2*>(outh + row_off + eb * 16) = r2;
            }
        }
    }
}

// Column sums of the attention probabilities (Sec. 3.3.1, the tensor D; Alg. 4):
//   D[b,h,i,j] = sum over the rows q of chunk i of exp(scale*s_qj - m_q) / l_q
// with (m_q, l_q) either from the dense attention pass of the same step (exact sums) or
// carried over from an earlier step (the stale-normaliser approximation of App. B.2).  Scores are produced as
// S = Q K^T (queries on the rows of the MFMA result), so that the sum over the
// chunk's queries is a sum over a lane's registers, the wave's four 16-lane
// rows and the workgroup's four waves.
struct ColsumParams {
    const uint16_t* q;
    const uint16_t* k;
    const float* row_m;
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
    constexpr int NI = kColsumTileRows / (RPI * 4);
    constexpr int TILE = kColsumTileRows * ROWB;
    __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * TILE];
    __shared__ float s_part[2][4][kColsumTileRows];

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
            m2v[qb][r] = ok ? p.row_m[bh * p.N + row0 + qr] * 1.4426950408889634f : 0.f;
            il[qb][r] = ok ? 1.f / p.row_l[bh * p.N + row0 + qr] : 0.f;
        }
    }
    const int koff = l16 * ROWB + ((g ^ swizzle<E>(l16)) * 16);
    const int grow0 = w * RPI + lane / CH;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (uint32_t)w * 1024u);
    const int ntiles = (p.N + kColsumTileRows - 1) / kColsumTileRows;

    auto gather = [&](int t, int stage) {
#pragma unroll
        for (int i = 0; i < NI; i++) {
            int row = grow0 + 4 * RPI * i;
            int pos = min(t * kColsumTileRows + row, p.N - 1);
            uint32_t goff = (uint32_t)pos * ROWB + (uint32_t)(((lane % CH) ^ swizzle<E>(row)) * 16);
            load_global_to_lds_16B(kh, goff, lds0 + (uint32_t)(stage * TILE + i * 4096));
        }
    };
    auto flush = [&](int t) {  // sums of tile t: four waves' partials -> global
        if (tid < kColsumTileRows) {
            int j = t * kColsumTileRows + tid;
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

template <int E, int NQB, int NWAVES, int MODE = kColumnList>
static int32_t launch_attn_variant(const AttnParams& p, int64_t units, hipStream_t s) {
    constexpr int lds = kStages * 2 * kTileRows * E * 2;
    // set at every launch: the attribute is kept per device, and a flag remembered here would be neither
    // per device nor safe between host threads
    if (hipFuncSetAttribute((const void*)attn_sparse_delta_kernel<E, NQB, NWAVES, MODE>,
                            hipFuncAttributeMaxDynamicSharedMemorySize, lds) != hipSuccess)
        return CHIPMUNK_ERR_LAUNCH;
    hipLaunchKernelGGL((attn_sparse_delta_kernel<E, NQB, NWAVES, MODE>), dim3((unsigned)units), dim3(64 * NWAVES), lds, s, p);
    return launch_status();
}

static int32_t launch_attn(const AttnParams& p, int E, int64_t units, hipStream_t s) {
    if (!p.idx) {
        if (E == 128 && p.c == 192) return launch_attn_variant<128, 3, 4, kEveryColumn>(p, units, s);
        if (E == 128 && p.c == 128) return launch_attn_variant<128, 2, 4, kEveryColumn>(p, units, s);
        if (E == 64 && p.c == 192) return launch_attn_variant<64, 3, 4, kEveryColumn>(p, units, s);
        return launch_attn_variant<64, 2, 4, kEveryColumn>(p, units, s);
    }
    if (E == 128 && p.c == 192) return launch_attn_variant<128, 3, 4>(p, units, s);
    if (E == 128 && p.c == 128) return launch_attn_variant<128, 2, 4>(p, units, s);
    if (E == 64 && p.c == 192) return launch_attn_variant<64, 3, 4>(p, units, s);
    return launch_attn_variant<64, 2, 4>(p, units, s);
}

static int32_t launch_attn_fused(const AttnParams& p, int E, int64_t units, hipStream_t s) {
    if (E == 128 && p.c == 192) return launch_attn_variant<128, 3, 4, kFusedDense>(p, units, s);
    if (E == 128 && p.c == 128) return launch_attn_variant<128, 2, 4, kFusedDense>(p, units, s);
    if (E == 64 && p.c == 192) return launch_attn_variant<64, 3, 4, kFusedDense>(p, units, s);
    return launch_attn_variant<64, 2, 4, kFusedDense>(p, units, s);
}

static int32_t launch_attn_blocks(const AttnParams& p, int E, int64_t units, hipStream_t s) {
    if (E == 128 && p.c == 192) return launch_attn_variant<128, 3, 4, kBlockList>(p, units, s);
    if (E == 128 && p.c == 128) return launch_attn_variant<128, 2, 4, kBlockList>(p, units, s);
    if (E == 64 && p.c == 192) return launch_attn_variant<64, 3, 4, kBlockList>(p, units, s);
    return launch_attn_variant<64, 2, 4, kBlockList>(p, units, s);
}

static int32_t launch_colsum(const ColsumParams& cp, int E, int64_t units, hipStream_t s) {
    dim3 grid((unsigned)units), block(256);
    if (E == 128 && cp.c == 192) hipLaunchKernelGGL((attn_colsum_kernel<128, 3>), grid, block, 0, s, cp);
    else if (E == 128 && cp.c == 128) hipLaunchKernelGGL((attn_colsum_kernel<128, 2>), grid, block, 0, s, cp);
    else if (E == 64 && cp.c == 192) hipLaunchKernelGGL((attn_colsum_kernel<64, 3>), grid, block, 0, s, cp);
    else hipLaunchKernelGGL((attn_colsum_kernel<64, 2>), grid, block, 0, s, cp);
    return launch_status();
}

// Shape rules common to the attention entry points.  Offsets of K/V rows inside one head are 32-bit byte offsets.
static int32_t check_attn_shapes(int B, int H, int N, int E, int c, float softmax_scale) {
    if (B < 1 || H < 1 || N < 1) return CHIPMUNK_ERR_SHAPE;
    if (!is_positive_finite_scalar(softmax_scale)) return CHIPMUNK_ERR_SHAPE;
    if (E != 64 && E != 128) return CHIPMUNK_ERR_UNSUPPORTED;
    if (c != 128 && c != 192) return CHIPMUNK_ERR_UNSUPPORTED;
    if ((int64_t)N * E * 2 >= (1LL << 32)) return CHIPMUNK_ERR_SHAPE;
    if ((int64_t)B * H * ((N + c - 1) / c) > 0x7fffffffLL) return CHIPMUNK_ERR_SHAPE;
    return CHIPMUNK_OK;
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
    if (k_stride < 0 || !is_finite_scalar(o_scale)) return CHIPMUNK_ERR_SHAPE;
    if (int32_t st = check_attn_shapes(B, H, N, E, c, softmax_scale)) return st;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(base) ||
        !aligned16(idx) || !aligned16(counts))
        return CHIPMUNK_ERR_ALIGN;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = base; p.out = out; p.idx = idx; p.counts = counts;
    p.row_m = nullptr; p.row_l = nullptr;
    p.prev_m = nullptr; p.prev_l = nullptr; p.colsum = nullptr; p.ld_colsum = 0;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = k_stride;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = o_scale;
    return launch_attn(p, E, units, (hipStream_t)stream);
}

extern "C" int32_t chipmunk_attn_block_sparse_delta(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                                    const int32_t* blocks, const int32_t* block_counts,
                                                    const uint16_t* base, uint16_t* out, int B, int H, int N,
                                                    int E, int c, int kb_stride, float softmax_scale,
                                                    float o_scale, void* stream) {
    if (!q || !k || !v || !out || !blocks || !block_counts || !base) return CHIPMUNK_ERR_NULL;
    if (kb_stride < 0 || !is_finite_scalar(o_scale)) return CHIPMUNK_ERR_SHAPE;
    if (int32_t st = check_attn_shapes(B, H, N, E, c, softmax_scale)) return st;
    if ((int64_t)kb_stride * kBlockColumns > 0x7fffffffLL) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(base) ||
        (reinterpret_cast<uintptr_t>(blocks) & 3u) || (reinterpret_cast<uintptr_t>(block_counts) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = base; p.out = out; p.idx = blocks; p.counts = block_counts;
    p.row_m = nullptr; p.row_l = nullptr;
    p.prev_m = nullptr; p.prev_l = nullptr; p.colsum = nullptr; p.ld_colsum = 0;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = kb_stride;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = o_scale;
    return launch_attn_blocks(p, E, units, (hipStream_t)stream);
}

extern "C" size_t chipmunk_attn_dense_workspace_bytes(int B, int H, int N) {
    if (B < 1 || H < 1 || N < 1) return 0;
    return (size_t)B * H * N * 2 * sizeof(float);
}

extern "C" int32_t chipmunk_attn_dense(const uint16_t* q, const uint16_t* k, const uint16_t* v, uint16_t* out,
                                       float* colsum, int64_t ld_colsum, int B, int H, int N, int E, int c,
                                       float softmax_scale, void* ws, size_t ws_bytes, void* stream) {
    if (!q || !k || !v || !out) return CHIPMUNK_ERR_NULL;
    if (int32_t st = check_attn_shapes(B, H, N, E, c, softmax_scale)) return st;
    if (colsum && ld_colsum < N) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(colsum) || !aligned16(ws) ||
        (colsum && (ld_colsum % 4) != 0))
        return CHIPMUNK_ERR_ALIGN;
    if (colsum && (!ws || ws_bytes < chipmunk_attn_dense_workspace_bytes(B, H, N))) return CHIPMUNK_ERR_WORKSPACE;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    hipStream_t s = (hipStream_t)stream;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = nullptr; p.out = out; p.idx = nullptr; p.counts = nullptr;
    p.row_m = colsum ? (float*)ws : nullptr;
    p.row_l = colsum ? (float*)ws + (int64_t)B * H * N : nullptr;
    p.prev_m = nullptr; p.prev_l = nullptr; p.colsum = nullptr; p.ld_colsum = 0;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = 0;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = 1.f;
    int32_t st = launch_attn(p, E, units, s);
    if (st != CHIPMUNK_OK || !colsum) return st;
    ColsumParams cp;
    cp.q = q; cp.k = k; cp.row_m = p.row_m; cp.row_l = p.row_l; cp.colsum = colsum; cp.ld = ld_colsum;
    cp.N = N; cp.NB = NB; cp.c = c; cp.sl2 = p.sl2;
    return launch_colsum(cp, E, units, s);
}

extern "C" int32_t chipmunk_attn_colsum_stale(const uint16_t* q, const uint16_t* k, const float* prev_m,
                                              const float* prev_l, float* colsum, int64_t ld_colsum, int B, int H,
                                              int N, int E, int c, float softmax_scale, void* stream) {
    if (!q || !k || !prev_m || !prev_l || !colsum) return CHIPMUNK_ERR_NULL;
    if (int32_t st = check_attn_shapes(B, H, N, E, c, softmax_scale)) return st;
    if (ld_colsum < N) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(colsum) || (ld_colsum % 4) != 0 ||
        (reinterpret_cast<uintptr_t>(prev_m) & 3u) || (reinterpret_cast<uintptr_t>(prev_l) & 3u))
        return CHIPMUNK_ERR_ALIGN;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    ColsumParams cp;
    cp.q = q; cp.k = k; cp.row_m = prev_m; cp.row_l = prev_l; cp.colsum = colsum; cp.ld = ld_colsum;
    cp.N = N; cp.NB = NB; cp.c = c; cp.sl2 = softmax_scale * 1.4426950408889634f;
    return launch_colsum(cp, E, units, (hipStream_t)stream);
}

extern "C" int32_t chipmunk_attn_dense_colsum_stale(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                                    uint16_t* out, const float* prev_m, const float* prev_l,
                                                    float* colsum, int64_t ld_colsum, float* new_m, float* new_l,
                                                    int B, int H, int N, int E, int c, float softmax_scale,
                                                    void* stream) {
    if (!q || !k || !v || !out || !prev_m || !prev_l || !colsum) return CHIPMUNK_ERR_NULL;
    if ((new_m == nullptr) != (new_l == nullptr)) return CHIPMUNK_ERR_NULL;
    if (int32_t st = check_attn_shapes(B, H, N, E, c, softmax_scale)) return st;
    if (ld_colsum < N) return CHIPMUNK_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(colsum) || (ld_colsum % 4) != 0)
        return CHIPMUNK_ERR_ALIGN;
    for (const float* f : {prev_m, prev_l, (const float*)new_m, (const float*)new_l})
        if (reinterpret_cast<uintptr_t>(f) & 3u) return CHIPMUNK_ERR_ALIGN;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    AttnParams p;
    p.q = q; p.k = k; p.v = v; p.base = nullptr; p.out = out; p.idx = nullptr; p.counts = nullptr;
    p.row_m = new_m; p.row_l = new_l;
    p.prev_m = prev_m; p.prev_l = prev_l; p.colsum = colsum; p.ld_colsum = ld_colsum;
    p.N = N; p.NB = NB; p.c = c; p.k_stride = 0;
    p.sl2 = softmax_scale * 1.4426950408889634f;
    p.o_scale = 1.f;
    return launch_attn_fused(p, E, units, (hipStream_t)stream);
}
