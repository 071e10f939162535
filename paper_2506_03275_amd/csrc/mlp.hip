// Column-sparse delta MLP (Sec. 3.3.2 "Sparse Delta Steps", App. B.3.1, Alg. 6),
// the dense MLP of a dense step (Alg. 5) and the token-merged pre-activation
// (Alg. 7) for gfx950.
//
// GEMM1  pre[tok, s] = <x[tok], w1[idx[s]]>: one workgroup owns (token chunk,
//        128 selected neurons).  The x tile and the gathered w1 rows stream
//        through LDS (asynchronous 16-byte loads, three tile buffers: two
//        contraction steps in flight while one is consumed, K tile 64)
//        into bf16 MFMA 32x32x16.  Epilogue: bias, activation, rounding to
//        bf16, a transpose through LDS to the neuron-major layout of a_cache,
//        then per 8 consecutive tokens of one neuron: read the cached
//        activation, write the new one, write delta^T to the workspace.  Each
//        (chunk, neuron) cell has one writer: no atomics.
// GEMM2  o_cache[tok, :] += sum_s delta[tok, s] * w2[idx[s], :]: one workgroup
//        owns (token chunk, 128 output columns) and walks the selected rows in
//        tiles of 64.  Both operands are stored with the contraction index as
//        the slow axis (delta^T rows, w2 rows), so both come out of LDS through
//        the transposing 64-bit read.  Epilogue: fp32 tile through LDS, add to
//        the cached output in fp32, round once, store in 256-byte runs.
// The dense MLP is the same two kernels with "every neuron selected": GEMM1
// writes a_cache only and GEMM2 reads its A operand from a_cache and adds b2.
#include "common.h"

#include <mutex>
#include <type_traits>

namespace chipmunk {

constexpr int kBN = 128;  // neurons (GEMM1) or output columns (GEMM2) per workgroup
constexpr int kBK = 64;   // contraction tile

enum Gemm1Mode { kSparseDelta = 0, kDenseAct = 1, kPlainF32 = 2 };

// Workgroups are dispatched to the eight XCDs round-robin by linear id, and each
// XCD has its own L2.  The tiles of one token chunk share that chunk's x rows
// (GEMM1) or delta^T rows (GEMM2), so they are mapped to ids that are congruent
// modulo 8: chunk u runs on XCD u % 8, its column tiles back to back.
// Returns false for the padding ids of the last group of eight chunks.
__device__ __forceinline__ bool xcd_tile_of_block(int col_tiles, int units, int* unit, int* col_tile) {
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int u = (slot / col_tiles) * 8 + xcd;
    *unit = u;
    *col_tile = slot % col_tiles;
    return u < units;
}
static int xcd_grid_size(int col_tiles, int units) { return ((units + 7) / 8) * 8 * col_tiles; }

// The dense forms (every neuron selected) share the weight tiles between chunks as well, and a weight tile is as
// large as a chunk's rows: here 8 chunks x 8 column tiles of one XCD are mapped to 64 consecutive slots, so that what
// runs side by side on an XCD reads 8 weight tiles and 8 row tiles, each eight times, instead of 64 weight tiles once.
// Chunks and column tiles are padded to multiples of 8 per XCD; padding ids return false.
__device__ __forceinline__ bool xcd_tile_of_block_grouped(int col_tiles, int units, int* unit, int* col_tile) {
    const int id = blockIdx.x;
    const int xcd = id & 7, slot = id >> 3;
    const int ctb_count = (col_tiles + 7) >> 3;          // blocks of 8 column tiles
    const int ct8 = slot & 7, lc8 = (slot >> 3) & 7;
    const int rest = slot >> 6;                          // = group of 8 local chunks * ctb_count + column-tile block
    const int g = rest / ctb_count, ctb = rest - g * ctb_count;
    const int u = (g * 8 + lc8) * 8 + xcd;               // local chunk g*8+lc8 of this XCD
    const int ct = ctb * 8 + ct8;
    *unit = u;
    *col_tile = ct;
    return u < units && ct < col_tiles;
}
static int xcd_grid_size_grouped(int col_tiles, int units) {
    const int local = (units + 7) / 8;                   // chunks per XCD
    return ((local + 7) / 8) * ((col_tiles + 7) / 8) * 64 * 8;
}


// ACT is a template argument so that a tile's activations are straight-line code: with the form chosen by a
// run-time branch inside, every element became a basic block of its own and its dozen dependent instructions
// ran one after the other.
template <int ACT>
__device__ __forceinline__ float gelu(float x) {
    if (ACT == CHIPMUNK_ACT_GELU_ERF) return 0.5f * x * (1.f + erff(x * 0.70710678118654752f));
    // tanh form: 0.5 x (1 + tanh(u)) = x / (1 + exp(-2u)),  u = sqrt(2/pi) (x + 0.044715 x^3)
    float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(-2.885390081777927f * u));  // v_rcp_f32: 1 ulp, the result is rounded to bf16
}

struct Gemm1Params {
    const uint16_t* x;       // [B, N, ldx] rows of K elements
    const uint16_t* w1;      // [F, D]
    const uint16_t* b1;      // [F] or null
    const int32_t* idx;      // [units, k_stride] or null (dense)
    const int32_t* counts;   // [units] or null
    uint16_t* a_cache;       // [B, F, a_ld]
    uint16_t* delta_t;       // workspace [units, k_pad, BM]
    uint16_t* act_t;         // null, or workspace [units, k_pad, BM]: the new activations go here (same layout as
                             // delta_t) instead of into a_cache; the second GEMM's launch writes them back
    float* out_f32;          // kPlainF32: [B*N, F]
    int64_t a_ld;
    int N, NB, D, F, K, ldx; // K = contraction length (D, or 2D for the split-precision scores GEMM)
    int k_stride, k_pad, act;
    int col_tiles, units;    // launch geometry (see xcd_tile_of_block)
    int ksplit;              // kPlainF32 only: the contraction is cut in ksplit pieces, one workgroup each,
                             // whose partial results go to out_f32 + piece * N * F (summed by a second kernel)
};

// NS tile buffers: NS - 1 contraction steps are in flight while one is consumed.  The column-sparse and the dense
// form run with three (120 KB, one workgroup per CU): measured against two buffers and two workgroups per CU,
// which keep the same number of bytes in flight, the MLP delta takes 11 % less time and the dense MLP 9 % less.
// The scores GEMM (few, short workgroups) keeps two.
template <int BM, int MODE, int NS, bool LOADER>
__global__ __launch_bounds__(LOADER ? 320 : 256, LOADER ? 1 : 2) void mlp_gemm1_kernel(Gemm1Params p) {
    // LOADER: a fifth wave issues every tile transfer of the workgroup; the four product waves issue none.  A wave
    // issues in order, so a transfer that waits for room in the memory pipeline holds up the products behind it.
    // The loader wave takes part in every barrier of the kernel and in nothing else.
    constexpr int VW = LOADER ? 4 : 1;             // waves whose share of the transfers one issuing wave carries
    constexpr int MT = BM / 64;                    // 32-row MFMA tiles per wave (wave tile = BM/2 x 64)
    constexpr int XT = BM * 128;                   // bytes of the x tile  [BM][64] bf16
    constexpr int WT = kBN * 128;                  // bytes of the w1 tile [128][64] bf16
    constexpr int STAGE = XT + WT;
    constexpr int NIX = BM / 32;                   // 16-byte loads per lane for the x tile
    constexpr int NIW = kBN / 32;
    constexpr int TS = BM * 2 + 16;                // row stride of the transposed epilogue tile
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];
    __shared__ int32_t s_neuron[kBN];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const bool loader = LOADER && w == 4;          // wave-uniform
    const int wm = w >> 1, wn = w & 1;
    const int l32 = lane & 31, h = lane >> 5;

    int unit, col_tile, piece = 0;                 // unit = (batch, token chunk)
    if (MODE == kPlainF32) {  // few row blocks: plain order, spread over every XCD
        col_tile = blockIdx.x % p.col_tiles;
        unit = (blockIdx.x / p.col_tiles) % p.units;
        piece = blockIdx.x / (p.col_tiles * p.units);
    } else if (MODE == kDenseAct ? !xcd_tile_of_block_grouped(p.col_tiles, p.units, &unit, &col_tile)
                                 : !xcd_tile_of_block(p.col_tiles, p.units, &unit, &col_tile)) {
        return;
    }
    const int b = unit / p.NB, chunk = unit % p.NB;
    const int row0 = chunk * BM;
    const int col0 = col_tile * kBN;
    const int count = p.counts ? min(p.counts[unit], p.k_stride) : p.F;   // clamped like the indices below: a bad
                                                                          // entry must not leave the tensors
    if (col0 >= count && MODE != kSparseDelta) return;
    if (MODE == kSparseDelta && col0 >= ((count + kBK - 1) / kBK) * kBK) return;  // nothing to compute or to zero

    // neuron of each of the 128 columns of this tile (clamped: columns at or beyond count
    // compute a duplicate that is never stored)
    if (tid < kBN) {
        int s = col0 + tid;
        int last = max(count - 1, 0);
        int f = p.idx ? min(max(p.idx[(int64_t)unit * p.k_stride + min(s, last)], 0), p.F - 1) : min(s, last);
        s_neuron[tid] = f;
    }
    __syncthreads();

    // per-lane source offsets (bytes) of the asynchronous tile loads; the K offset is uniform
    uint32_t xoff[NIX * VW], woff[NIW * VW];
#pragma unroll
    for (int i = 0; i < NIX; i++)
#pragma unroll
        for (int v = 0; v < VW; v++) {
            int row = (i * 4 + (LOADER ? v : w)) * 8 + (lane >> 3);
            int chunk16 = (lane & 7) ^ ((row >> 1) & 7);
            int tok = min(row0 + row, p.N - 1);
            xoff[i * VW + v] = (uint32_t)tok * (uint32_t)(p.ldx * 2) + chunk16 * 16;
        }
#pragma unroll
    for (int i = 0; i < NIW; i++)
#pragma unroll
        for (int v = 0; v < VW; v++) {
            int row = (i * 4 + (LOADER ? v : w)) * 8 + (lane >> 3);
            int chunk16 = (lane & 7) ^ ((row >> 1) & 7);
            woff[i * VW + v] = (uint32_t)s_neuron[row] * (uint32_t)(p.D * 2) + chunk16 * 16;
        }
    const uint16_t* xb = p.x + (int64_t)b * p.N * p.ldx;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (LOADER ? 0u : (uint32_t)w * 1024u));

    // One of the transfers that bring contraction step kt into buffer `stage`.  Without a loader wave the main loop
    // issues a wave's NIX + NIW two by two between its products: requested in one burst after the barrier they
    // queue up in the memory pipeline while the wave issues nothing else.
    auto issue_piece = [&](int kt, int stage, int j) {   // j < (NIX + NIW) * VW; piece (i, v) = (j / VW, j % VW)
        const int i = j / VW, v = j % VW;
        if (i < NIX) {
            load_global_to_lds_16B(xb + kt * kBK, xoff[j], lds0 + stage * STAGE + i * 4096 + v * 1024);
        } else {
            const uint16_t* ws = p.w1 + (kt * kBK) % p.D;   // the scores GEMM walks w1's row twice (hi and lo halves of A)
            load_global_to_lds_16B(ws, woff[j - NIX * VW], lds0 + stage * STAGE + XT + (i - NIX) * 4096 + v * 1024);
        }
    };
    static_assert(NIX + NIW <= 4 * MT, "one transfer per pair of products");

    f32x16 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int nt = 0; nt < 2; nt++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[mt][nt][r] = 0.f;

    // LDS read offsets: row l32 of a 32-row tile, 16-byte chunk (2*ks + h) ^ swizzle(row)
    const int sw = (l32 >> 1) & 7;
    const int aoff = (wm * (BM / 2) + l32) * 128 + ((h ^ sw) * 16);
    const int boff = XT + (wn * 64 + l32) * 128 + ((h ^ sw) * 16);

    const int ktiles_all = p.K / kBK;
    const int kt_begin = MODE == kPlainF32 ? (int)((int64_t)ktiles_all * piece / p.ksplit) : 0;
    const int kt_end = MODE == kPlainF32 ? (int)((int64_t)ktiles_all * (piece + 1) / p.ksplit) : ktiles_all;
    constexpr int NP = NIX + NIW;
    if (!LOADER || loader) {
#pragma unroll
        for (int st = 0; st < NS - 1; st++)
#pragma unroll
            for (int j = 0; j < NP * VW; j++) issue_piece(min(kt_begin + st, max(kt_end - 1, kt_begin)), st, j);
    }
    int stage = 0;
    static_assert((NS - 2) * NP * VW < 64, "the transfer counter has six bits");
    if (loader) {
        for (int kt = kt_begin; kt < kt_end; kt++) {
            wait_vmem_at_most<(NS - 2) * NP * VW>();
            __syncthreads();
            const int kt_next = min(kt + NS - 1, kt_end - 1);
            const int fill = (stage + NS - 1) % NS;
#pragma unroll
            for (int j = 0; j < NP * VW; j++) issue_piece(kt_next, fill, j);
            stage = stage + 1 == NS ? 0 : stage + 1;
        }
        wait_all_memory();                 // the transfers must have landed before the epilogue reuses the buffers
        lds_accesses_then_barrier();       // the two barriers of the epilogue
        lds_accesses_then_barrier();
        return;
    }
    for (int kt = kt_begin; kt < kt_end; kt++) {
        // The transfers complete in the order they were issued: this step's tiles have landed when no more than
        // the pieces of the NS - 2 younger steps are outstanding.
        wait_vmem_at_most<(NS - 2) * NP>();
        __syncthreads();
        // NS - 1 steps ahead; past the end the last step is fetched again into a buffer nobody reads
        const int kt_next = min(kt + NS - 1, kt_end - 1);
        const int fill = (stage + NS - 1) % NS;    // the buffer the step before this one has just left
        const uint8_t* sb = smem + stage * STAGE;
        // The operands of contraction sub-step ks + 1 are requested ahead of the products of sub-step ks (two
        // register sets): with one wave per SIMD nothing else covers the LDS latency between a read and its product.
        bf16x8 aop[2][MT], bop[2][2];
        auto read_operands = [&](int ks, int set) {
#pragma unroll
            for (int nt = 0; nt < 2; nt++)
                bop[set][nt] = *reinterpret_cast<const bf16x8*>(sb + nt * 32 * 128 + (boff ^ (32 * ks)));
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
                aop[set][mt] = *reinterpret_cast<const bf16x8*>(sb + mt * 32 * 128 + (aoff ^ (32 * ks)));
        };
        read_operands(0, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, MT + 2, 0);
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            if (ks + 1 < 4) {
                read_operands(ks + 1, (ks + 1) & 1);
                __builtin_amdgcn_sched_group_barrier(0x100, MT + 2, 0);   // the reads lead the block
            }
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
#pragma unroll
                for (int nt = 0; nt < 2; nt++)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop[ks & 1][mt], bop[ks & 1][nt], acc[mt][nt], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                if (!LOADER) {
                    const int slot = ks * MT + mt;
                    if (2 * slot < NP) issue_piece(kt_next, fill, 2 * slot);
                    if (2 * slot + 1 < NP) issue_piece(kt_next, fill, 2 * slot + 1);
                }
            }
        }
        stage = stage + 1 == NS ? 0 : stage + 1;
    }

    wait_all_memory();  // an empty piece of a split contraction still has its first tile in flight

    if (MODE == kPlainF32) {
        // out[row, col] fp32; a lane holds one column and 4 consecutive rows per register group
#pragma unroll
        for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int nt = 0; nt < 2; nt++) {
                int col = col0 + wn * 64 + nt * 32 + l32;
#pragma unroll
                for (int r = 0; r < 16; r++) {
                    int row = row0 + wm * (BM / 2) + mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                    if (row < p.N && col < p.F)
                        p.out_f32[((int64_t)piece * p.N + row) * p.F + col] = acc[mt][nt][r];
                }
            }
        return;
    }

    // ---- epilogue: bias, activation, bf16, transpose to [neuron][token] through LDS ----
    constexpr int CPR = BM / 8;                  // 16-byte chunks (8 tokens) per neuron row
    constexpr int ITEMS = kBN * CPR / 256;       // (neuron, 8 tokens) cells per thread
    static_assert(kBN * CPR % 256 == 0, "the tile's cells must divide over the threads");
    // The cached activations of this thread's cells are requested here, ahead of the activation arithmetic and
    // the transposition, so that their latency is paid once and in the shadow of that work.  One 16-byte load per
    // cell whatever the case (cells past the end of the row or of the list read a valid address and are not
    // used): a_ld is a multiple of 8 and at least N, so a cell that starts below N ends inside its row.
    // bias of the lane's two neuron columns: requested first (the activation arithmetic waits for these only) and
    // without a branch (w1 stands in as a valid address when there is no bias)
    const uint16_t* bias_src = p.b1 ? p.b1 : p.w1;
    uint16_t bias_raw[2];
#pragma unroll
    for (int nt = 0; nt < 2; nt++) bias_raw[nt] = bias_src[s_neuron[wn * 64 + nt * 32 + l32]];
    u32x4 old8[ITEMS];
    uint16_t* cell[ITEMS];   // the thread's cells in a_cache (token clamped to the row's start where the chunk ends early)
#pragma unroll
    for (int n = 0; n < ITEMS; n++) {
        const int item = tid + n * 256;
        const int nl = item / CPR, ch = item - nl * CPR;
        const int tok0 = row0 + ch * 8;
        cell[n] = p.a_cache + ((int64_t)b * p.F + s_neuron[nl]) * p.a_ld + (tok0 < p.N ? tok0 : 0);
        if (MODE == kSparseDelta) old8[n] = *reinterpret_cast<const u32x4*>(cell[n]);
    }
    lds_accesses_then_barrier();  // every wave is done with the stage buffers
    float bias[2];
#pragma unroll
    for (int nt = 0; nt < 2; nt++) bias[nt] = p.b1 ? bf16_bits_to_float(bias_raw[nt]) : 0.f;
    auto activate_tile = [&](auto form) {
        constexpr int ACT = decltype(form)::value;
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
            int nl = wn * 64 + nt * 32 + l32;
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int rg = 0; rg < 4; rg++) {
                    int tl = wm * (BM / 2) + mt * 32 + rg * 8 + h * 4;
                    float a0 = gelu<ACT>(acc[mt][nt][rg * 4 + 0] + bias[nt]);
                    float a1 = gelu<ACT>(acc[mt][nt][rg * 4 + 1] + bias[nt]);
                    float a2 = gelu<ACT>(acc[mt][nt][rg * 4 + 2] + bias[nt]);
                    float a3 = gelu<ACT>(acc[mt][nt][rg * 4 + 3] + bias[nt]);
                    u32x2 v = {pack_bf16x2(a0, a1), pack_bf16x2(a2, a3)};
                    *reinterpret_cast<u32x2*>(smem + nl * TS + tl * 2) = v;
                }
        }
    };
    if (p.act == CHIPMUNK_ACT_GELU_ERF) activate_tile(std::integral_constant<int, CHIPMUNK_ACT_GELU_ERF>{});
    else activate_tile(std::integral_constant<int, CHIPMUNK_ACT_GELU_TANH>{});
    lds_accesses_then_barrier();
    // The cells are handled in three sweeps (read the transposed tile, form the deltas, store) of straight-line
    // code: in one loop with a branch per cell every cell waited for its own LDS reads, and the compiler, which
    // counts a wait as if no store had been issued on the way, made it wait for the stores of the cells before.
    u32x4 a8[ITEMS];
#pragma unroll
    for (int n = 0; n < ITEMS; n++) {
        const int item = tid + n * 256;
        const int nl = item / CPR, ch = item - nl * CPR;
        a8[n] = *reinterpret_cast<const u32x4*>(smem + nl * TS + ch * 16);
    }
    if (MODE == kSparseDelta) {
        // the cached activations, requested before the activation arithmetic, are taken as arrived in one wait
#pragma unroll
        for (int n = 0; n < ITEMS; n++) asm volatile("" ::"v"(old8[n]), "v"(a8[n]));
        uint16_t* dunit = p.delta_t + (int64_t)unit * p.k_pad * BM;
#pragma unroll
        for (int n = 0; n < ITEMS; n++) {
            const int item = tid + n * 256;
            const int nl = item / CPR, ch = item - nl * CPR;
            const int s = col0 + nl;
            // tokens past N and padding rows of the contraction must read as zero in GEMM2
            const int nvalid = s < count ? min(8, p.N - (row0 + ch * 8)) : 0;
            u32x4 d8;
#pragma unroll
            for (int e2 = 0; e2 < 4; e2++) {
                float dlo = bf16_bits_to_float(a8[n][e2] & 0xffffu) - bf16_bits_to_float(old8[n][e2] & 0xffffu);
                float dhi = bf16_bits_to_float(a8[n][e2] >> 16) - bf16_bits_to_float(old8[n][e2] >> 16);
                if (2 * e2 >= nvalid) dlo = 0.f;
                if (2 * e2 + 1 >= nvalid) dhi = 0.f;
                d8[e2] = pack_bf16x2(dlo, dhi);
            }
            if (s < p.k_pad) *reinterpret_cast<u32x4*>(dunit + (s * BM + ch * 8)) = d8;
        }
    }
#pragma unroll
    for (int n = 0; n < ITEMS; n++) {
        const int item = tid + n * 256;
        const int nl = item / CPR, ch = item - nl * CPR;
        const int s = col0 + nl;
        const int nvalid = s < count ? min(8, p.N - (row0 + ch * 8)) : 0;
        if (MODE == kSparseDelta && p.act_t) {   // deferred write-back: one coalesced store, whole cell
            if (nvalid > 0) *reinterpret_cast<u32x4*>(p.act_t + ((int64_t)unit * p.k_pad + s) * BM + ch * 8) = a8[n];
        } else if (nvalid == 8) {
            *reinterpret_cast<u32x4*>(cell[n]) = a8[n];
        } else {  // the cells past N in the last chunk stay as they are
            for (int e = 0; e < nvalid; e++) cell[n][e] = (uint16_t)(a8[n][e >> 1] >> (16 * (e & 1)));
        }
    }
}

struct Gemm2Params {
    const uint16_t* a_t;     // sparse: delta^T workspace [units, k_pad, BM]; dense: a_cache [B, F, a_ld]
    const uint16_t* w2;      // [F, D]
    const uint16_t* bias;    // dense: b2 [D] or null
    const int32_t* idx;      // [units, k_stride] or null
    const int32_t* counts;   // [units] or null
    uint16_t* o;             // sparse: o_cache in/out; dense: out
    int64_t a_ld;
    int N, NB, D, F, k_stride, k_pad;
    int dense;
    int col_tiles, units;    // launch geometry (see xcd_tile_of_block)
    // Deferred cache write-back (App. B.3.3): workgroups with id >= tile_blocks, one per unit, copy the new
    // activations that the first GEMM left in act_t into a_cache while the tile workgroups of this launch compute.
    const uint16_t* act_t;   // null: no write-back workgroups
    uint16_t* a_cache;
    int tile_blocks;
};

template <int BM>
__device__ __forceinline__ int swizzle_at(int row) {  // for rows of BM tokens (BM*2 bytes)
    if (BM == 192) return (row & 2) << 1;
    return ((row & 3) << 2) | ((row >> 2) & 3);
}
__device__ __forceinline__ int swizzle_w2(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

template <int BM>
__global__ __launch_bounds__(256, 2) void mlp_gemm2_kernel(Gemm2Params p) {
    constexpr int MT = BM / 64;
    constexpr int RBA = BM * 2;                    // bytes per row of the A^T tile
    constexpr int CPA = BM / 8;                    // 16-byte chunks per A^T row
    constexpr int AT = kBK * RBA;                  // A^T tile bytes [64][BM]
    constexpr int WT = kBK * 256;                  // w2 tile bytes  [64][128]
    constexpr int STAGE = AT + WT;
    constexpr int NIA = kBK * CPA / 256;           // loads per lane, A^T tile
    constexpr int NIW = kBK * 16 / 256;            // loads per lane, w2 tile
    constexpr int CS = 128 * 4 + 32;               // row stride (bytes) of the fp32 epilogue tile
    extern __shared__ __attribute__((aligned(1024))) uint8_t smem[];

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    const int l16 = lane & 15, mb = (lane >> 4) & 1, h = lane >> 5;

    if (p.act_t && (int)blockIdx.x >= p.tile_blocks) {
        // A write-back workgroup.  They have the highest ids, so they start when the tile workgroups' last round
        // leaves compute units free, and their memory traffic runs beside that round's products.
        const int u = (int)blockIdx.x - p.tile_blocks;
        const int ub = u / p.NB, urow0 = (u % p.NB) * BM;
        const int ucount = max(min(p.counts[u], p.k_stride), 0);
        constexpr int CPR = BM / 8;
        for (int item = tid; item < ucount * CPR; item += 256) {
            const int s = item / CPR, ch = item - s * CPR;
            const int tok0 = urow0 + ch * 8;
            const int nvalid = min(8, p.N - tok0);
            if (nvalid <= 0) continue;
            const int f = min(max(p.idx[(int64_t)u * p.k_stride + s], 0), p.F - 1);
            const u32x4 a8 = *reinterpret_cast<const u32x4*>(p.act_t + ((int64_t)u * p.k_pad + s) * BM + ch * 8);
            uint16_t* arow = p.a_cache + ((int64_t)ub * p.F + f) * p.a_ld + tok0;
            if (nvalid == 8) {
                *reinterpret_cast<u32x4*>(arow) = a8;
            } else {  // the cells past N in the last chunk stay as they are
                for (int e = 0; e < nvalid; e++) arow[e] = (uint16_t)(a8[e >> 1] >> (16 * (e & 1)));
            }
        }
        return;
    }
    int unit, col_tile;
    if (p.dense ? !xcd_tile_of_block_grouped(p.col_tiles, p.units, &unit, &col_tile)
                : !xcd_tile_of_block(p.col_tiles, p.units, &unit, &col_tile))
        return;
    const int b = unit / p.NB, chunk = unit % p.NB;
    const int row0 = chunk * BM;
    const int d0 = col_tile * kBN;
    const int count = p.counts ? min(p.counts[unit], p.k_stride) : p.F;
    if (count <= 0 && !p.dense) return;            // nothing selected: the cache stays as it is
    const int32_t* idxp = p.idx ? p.idx + (int64_t)unit * p.k_stride : nullptr;
    const int ktiles = (count + kBK - 1) / kBK;

    // A^T source: row (selected slot or neuron) -> tokens of this chunk
    const uint16_t* abase;
    int64_t a_row_stride;                          // elements between consecutive contraction rows
    if (p.dense) {
        abase = p.a_t + (int64_t)b * p.F * p.a_ld + row0;
        a_row_stride = p.a_ld;
    } else {
        abase = p.a_t + (int64_t)unit * p.k_pad * BM;
        a_row_stride = BM;
    }
    uint32_t aoff_g[NIA];
#pragma unroll
    for (int i = 0; i < NIA; i++) {
        int q = (i * 4 + w) * 64 + lane;           // linear 16-byte chunk of the tile
        int row = q / CPA, pos = q - row * CPA;
        int c16 = pos ^ swizzle_at<BM>(row);
        if (p.dense && row0 + c16 * 8 >= p.N) c16 = 0;  // tokens beyond N: any valid data, the rows are not stored
        aoff_g[i] = (uint32_t)((int64_t)row * a_row_stride * 2 + c16 * 16);
    }
    int wrow[NIW];
    uint32_t wchunk[NIW];
#pragma unroll
    for (int i = 0; i < NIW; i++) {
        wrow[i] = (i * 4 + w) * 4 + (lane >> 4);
        wchunk[i] = (uint32_t)(((lane & 15) ^ swizzle_w2(wrow[i])) * 16);
    }
    const uint16_t* w2b = p.w2 + d0;
    const uint32_t lds0 = __builtin_amdgcn_readfirstlane(lds_address(smem) + (uint32_t)w * 1024u);

    int cols[NIW];
    auto load_cols = [&](int kt) {
#pragma unroll
        for (int i = 0; i < NIW; i++) {
            int pos = min(kt * kBK + wrow[i], count - 1);
            cols[i] = idxp ? idxp[pos] : pos;
        }
    };
    // One of the NIA + NIW transfers of contraction step kt into buffer `stage` (issued one by one between the
    // products of the step before, not in one burst); the w2 pieces use the columns that load_cols brought.
    auto issue_piece = [&](int kt, int stage, int j) {
        if (j < NIA) {
            load_global_to_lds_16B(abase + (int64_t)kt * kBK * a_row_stride, aoff_g[j], lds0 + stage * STAGE + j * 4096);
        } else {
            const int i = j - NIA;
            load_global_to_lds_16B(w2b, (uint32_t)min(max(cols[i], 0), p.F - 1) * (uint32_t)(p.D * 2) + wchunk[i],
                                   lds0 + stage * STAGE + AT + i * 4096);
        }
    };
    static_assert(NIA + NIW <= 4 * MT, "one transfer per pair of products");

    f32x16 acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int nt = 0; nt < 2; nt++)
#pragma unroll
            for (int r = 0; r < 16; r++) acc[mt][nt][r] = 0.f;

    // Transposing reads.  For a k-step of 16 contraction rows, half h of the wave
    // takes rows 8h..8h+7 as two groups of 4; inside a block of 16 lanes, lane i
    // addresses row (i/4) of the group and 4 consecutive columns 4*(i%4).
    const int trow = 8 * h + (l16 >> 2);           // + 4*rd, + 16*ks
    const int tcol = 4 * (l16 & 3);                // element offset inside the 16-column block

    if (ktiles > 0) {
        load_cols(0);
#pragma unroll
        for (int j = 0; j < NIA + NIW; j++) issue_piece(0, 0, j);
        load_cols(min(1, ktiles - 1));
    }
    for (int kt = 0; kt < ktiles; kt++) {
        const int stage = kt & 1;
        wait_all_memory();
        __syncthreads();
        // the step after this one; past the end the last step is fetched once more into the buffer nobody reads
        const int kt_next = min(kt + 1, ktiles - 1);
        const uint8_t* sa = smem + stage * STAGE;
        const uint8_t* sw = sa + AT;
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            bf16x8 bop[2];
#pragma unroll
            for (int nt = 0; nt < 2; nt++) {
                short4v part[2];
#pragma unroll
                for (int rd = 0; rd < 2; rd++) {
                    int row = ks * 16 + trow + 4 * rd;
                    int col = wn * 64 + nt * 32 + mb * 16 + tcol;       // element column
                    int c16 = (col >> 3) ^ swizzle_w2(row);
                    part[rd] = lds_read_tr16(sw + row * 256 + c16 * 16 + (col & 7) * 2);
                }
                typedef __attribute__((ext_vector_type(8))) short short8v;
                bop[nt] = __builtin_bit_cast(bf16x8, (short8v)__builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7));
            }
#pragma unroll
            for (int mt = 0; mt < MT; mt++) {
                short4v part[2];
#pragma unroll
                for (int rd = 0; rd < 2; rd++) {
                    int row = ks * 16 + trow + 4 * rd;
                    int col = wm * (BM / 2) + mt * 32 + mb * 16 + tcol;  // token column
                    int c16 = (col >> 3) ^ swizzle_at<BM>(row);
                    part[rd] = lds_read_tr16(sa + row * RBA + c16 * 16 + (col & 7) * 2);
                }
                typedef __attribute__((ext_vector_type(8))) short short8v;
                bf16x8 aop = __builtin_bit_cast(bf16x8, (short8v)__builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int nt = 0; nt < 2; nt++)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aop, bop[nt], acc[mt][nt], 0, 0, 0);
                {
                    const int slot = ks * MT + mt;
                    if (2 * slot < NIA + NIW) issue_piece(kt_next, stage ^ 1, 2 * slot);
                    if (2 * slot + 1 < NIA + NIW) issue_piece(kt_next, stage ^ 1, 2 * slot + 1);
                }
            }
        }
        load_cols(min(kt + 2, ktiles - 1));   // for the transfers that the next step issues
    }
    wait_all_memory();  // the last step's transfers into the unused buffer must have landed before LDS is reused

    // ---- epilogue: fp32 tile through LDS, one half of the token rows at a time ----
    // What is added to (the cached output, or the bias of the dense form) is requested for both halves before the
    // tile goes through LDS: the reads are in flight behind the barriers instead of one round trip per item.
    const int l32 = lane & 31;
    constexpr int ITEMS = (BM / 2) * 32 / 256;     // 16-byte groups of four output columns per thread and half
    static_assert((BM / 2) * 32 % 256 == 0, "the half tile must divide over the threads");
    u32x2 old[2][ITEMS];
#pragma unroll
    for (int half = 0; half < 2; half++)
#pragma unroll
        for (int n = 0; n < ITEMS; n++) {
            const int item = tid + n * 256;
            const int tl = item >> 5, ch = item & 31;
            const int tok = row0 + half * (BM / 2) + tl;
            // one load per item whatever the case (a token past the end reads the last token's row, the dense form
            // without a bias reads the output buffer; neither value is used): branches here would make every
            // load wait for the one before
            const uint16_t* src = (p.dense && p.bias)
                                      ? p.bias + d0 + ch * 4
                                      : p.o + ((int64_t)b * p.N + min(tok, p.N - 1)) * p.D + d0 + ch * 4;
            old[half][n] = *reinterpret_cast<const u32x2*>(src);
        }
    const bool add_nothing = p.dense && !p.bias;
#pragma unroll
    for (int half = 0; half < 2; half++) {
        lds_accesses_then_barrier();
        if (wm == half) {
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int nt = 0; nt < 2; nt++)
#pragma unroll
                    for (int r = 0; r < 16; r++) {
                        int tl = mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                        int dl = wn * 64 + nt * 32 + l32;
                        *reinterpret_cast<float*>(smem + tl * CS + dl * 4) = acc[mt][nt][r];
                    }
        }
        lds_accesses_then_barrier();
        if (half == 0) {
            // Every value requested above is taken as arrived before the first store, in one wait.  The stores sit
            // in branches, so the waits the compiler counts per item assume that none was issued: left to the
            // loop, the second half's items would wait for the first half's stores.
#pragma unroll
            for (int hh = 0; hh < 2; hh++)
#pragma unroll
                for (int n = 0; n < ITEMS; n++) asm volatile("" ::"v"(old[hh][n]));
        }
        // two sweeps of straight-line code (read the staged tile, then merge and store): in one loop with the
        // store's branch inside, every item waited for its own LDS read
        f32x4 a4[ITEMS];
#pragma unroll
        for (int n = 0; n < ITEMS; n++) {
            const int item = tid + n * 256;
            a4[n] = *reinterpret_cast<const f32x4*>(smem + (item >> 5) * CS + (item & 31) * 16);
        }
#pragma unroll
        for (int n = 0; n < ITEMS; n++) {
            const int item = tid + n * 256;
            const int tl = item >> 5, ch = item & 31;
            const int tok = row0 + half * (BM / 2) + tl;
            uint16_t* orow = p.o + ((int64_t)b * p.N + tok) * p.D + d0 + ch * 4;
            const u32x2 o2 = add_nothing ? u32x2{0, 0} : old[half][n];
            float o0 = bf16_bits_to_float(o2[0] & 0xffffu) + a4[n][0];
            float o1 = bf16_bits_to_float(o2[0] >> 16) + a4[n][1];
            float o2f = bf16_bits_to_float(o2[1] & 0xffffu) + a4[n][2];
            float o3 = bf16_bits_to_float(o2[1] >> 16) + a4[n][3];
            u32x2 res = {pack_bf16x2(o0, o1), pack_bf16x2(o2f, o3)};
            if (tok < p.N) *reinterpret_cast<u32x2*>(orow) = res;
        }
    }
}

// Chunk means of x in split precision: mean = hi + lo with hi = bf16(mean),
// lo = bf16(mean - hi); out row = [hi(0..D-1) | lo(0..D-1)].  A workgroup owns
// (chunk, 512 columns): each wave sums a quarter of the chunk's rows for 64
// groups of 8 columns (16-byte reads), the four partial sums meet in LDS.
__global__ __launch_bounds__(256) void chunk_mean_kernel(const uint16_t* __restrict__ x, uint16_t* __restrict__ xm,
                                                         int N, int NB, int D, int c) {
    __shared__ float s_part[3][64][8];
    const int col_blocks = (D / 8 + 63) / 64;        // grid.x = units * col_blocks
    const int unit = blockIdx.x / col_blocks;
    const int b = unit / NB, chunk = unit % NB;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int col8 = (blockIdx.x % col_blocks) * 64 + lane;
    const bool live = col8 * 8 < D;
    const int r0 = chunk * c, r1 = min(N, r0 + c);
    float s[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (live) {
        for (int r = r0 + w; r < r1; r += 4) {
            u32x4 v = *reinterpret_cast<const u32x4*>(x + ((int64_t)b * N + r) * D + col8 * 8);
#pragma unroll
            for (int e = 0; e < 4; e++) {
                s[2 * e] += bf16_bits_to_float(v[e] & 0xffffu);
                s[2 * e + 1] += bf16_bits_to_float(v[e] >> 16);
            }
        }
    }
    if (w > 0) {
#pragma unroll
        for (int e = 0; e < 8; e++) s_part[w - 1][lane][e] = s[e];
    }
    __syncthreads();
    if (w > 0 || !live) return;
#pragma unroll
    for (int e = 0; e < 8; e++) s[e] += s_part[0][lane][e] + s_part[1][lane][e] + s_part[2][lane][e];
    const float inv = 1.f / (float)(r1 - r0);
    u32x4 hi4, lo4;
#pragma unroll
    for (int e = 0; e < 4; e++) {
        float m0 = s[2 * e] * inv, m1 = s[2 * e + 1] * inv;
        uint32_t hp = pack_bf16x2(m0, m1);
        hi4[e] = hp;
        lo4[e] = pack_bf16x2(m0 - bf16_bits_to_float(hp & 0xffffu), m1 - bf16_bits_to_float(hp >> 16));
    }
    uint16_t* orow = xm + (int64_t)unit * 2 * D;
    *reinterpret_cast<u32x4*>(orow + col8 * 8) = hi4;
    *reinterpret_cast<u32x4*>(orow + D + col8 * 8) = lo4;
}

// out[i] = sum over the pieces of a split contraction, in piece order (deterministic)
__global__ __launch_bounds__(256) void sum_pieces_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                         int64_t n4, int pieces) {
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n4) return;
    f32x4 acc = reinterpret_cast<const f32x4*>(part)[i];
    for (int pc = 1; pc < pieces; pc++) acc += reinterpret_cast<const f32x4*>(part)[pc * n4 + i];
    reinterpret_cast<f32x4*>(out)[i] = acc;
}

template <int BM, int MODE>
static int32_t launch_gemm1(Gemm1Params p, int col_tiles, int units, hipStream_t s) {
    p.col_tiles = col_tiles;
    p.units = units;
    constexpr int NS = MODE == kPlainF32 ? 2 : 3;
    constexpr bool LOADER = MODE != kPlainF32;
    constexpr int lds = NS * (BM * 128 + kBN * 128);
    // set at every launch: the attribute is kept per device (a flag remembered here would not be)
    if (hipFuncSetAttribute((const void*)mlp_gemm1_kernel<BM, MODE, NS, LOADER>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) !=
        hipSuccess)
        return CHIPMUNK_ERR_LAUNCH;
    const int grid = MODE == kPlainF32 ? col_tiles * units * p.ksplit
                     : MODE == kDenseAct ? xcd_grid_size_grouped(col_tiles, units)
                                         : xcd_grid_size(col_tiles, units);
    hipLaunchKernelGGL((mlp_gemm1_kernel<BM, MODE, NS, LOADER>), dim3(grid), dim3(LOADER ? 320 : 256), lds, s, p);
    return launch_status();
}

template <int BM>
static int32_t launch_gemm2(Gemm2Params p, int col_tiles, int units, hipStream_t s) {
    p.col_tiles = col_tiles;
    p.units = units;
    constexpr int stage = kBK * BM * 2 + kBK * 256;
    constexpr int epi = (BM / 2) * (128 * 4 + 32);
    constexpr int lds = 2 * stage > epi ? 2 * stage : epi;
    if (hipFuncSetAttribute((const void*)mlp_gemm2_kernel<BM>, hipFuncAttributeMaxDynamicSharedMemorySize, lds) !=
        hipSuccess)
        return CHIPMUNK_ERR_LAUNCH;
    p.tile_blocks = p.dense ? xcd_grid_size_grouped(col_tiles, units) : xcd_grid_size(col_tiles, units);
    const int grid = p.tile_blocks + (p.act_t ? units : 0);
    hipLaunchKernelGGL((mlp_gemm2_kernel<BM>), dim3((unsigned)grid), dim3(256), lds, s, p);
    return launch_status();
}

static int round_up(int v, int m) { return (v + m - 1) / m * m; }

static int32_t check_mlp_shapes(int B, int N, int D, int F, int c) {
    if (B < 1 || N < 1 || D < 1 || F < 1) return CHIPMUNK_ERR_SHAPE;
    if (c != 128 && c != 192) return CHIPMUNK_ERR_UNSUPPORTED;
    if (D % 128 != 0 || F % 64 != 0) return CHIPMUNK_ERR_UNSUPPORTED;
    if ((int64_t)N * D * 2 >= (1LL << 32) || (int64_t)F * D * 2 >= (1LL << 32)) return CHIPMUNK_ERR_SHAPE;
    if ((int64_t)B * ((N + c - 1) / c) * ((F + kBN - 1) / kBN + D / kBN) > 0x3fffffffLL) return CHIPMUNK_ERR_SHAPE;
    return CHIPMUNK_OK;
}

}  // namespace chipmunk

using namespace chipmunk;

extern "C" size_t chipmunk_mlp_workspace_bytes(int B, int N, int D, int F, int c, int k_stride) {
    if (check_mlp_shapes(B, N, D, F, c) != CHIPMUNK_OK || k_stride < 0 || k_stride > F) return 0;
    int64_t units = (int64_t)B * ((N + c - 1) / c);
    return (size_t)(units * round_up(k_stride > 0 ? k_stride : 1, kBN) * c * 2);
}

// pieces the scores GEMM's contraction is cut into, so that a small problem still fills the GPU
static int tile_mean_pieces(int units, int F) {
    int blocks = ((units + 127) / 128) * ((F + kBN - 1) / kBN);
    int pieces = 1;
    while (pieces < 16 && blocks * pieces < 768) pieces *= 2;
    return pieces;
}

// Workspace of the token-merged pre-activation with the contraction cut in `pieces`: the chunk means in split
// precision [units, 2 D] bf16 (rounded up to 256 bytes), then, with more than one piece, the pieces' partial
// results [pieces, units, F] fp32.  0 when the shapes are out of range.
static size_t tile_mean_bytes(int B, int N, int D, int F, int c, int pieces) {
    if (check_mlp_shapes(B, N, D, F, c) != CHIPMUNK_OK) return 0;
    const int64_t units = (int64_t)B * ((N + c - 1) / c);
    if (units > 0x7fffff || units * 2 * D * 2 >= (1LL << 32)) return 0;
    const size_t means = ((size_t)units * 2 * D * 2 + 255) / 256 * 256;
    return means + (pieces > 1 ? (size_t)pieces * units * F * sizeof(float) : 0);
}

extern "C" size_t chipmunk_mlp_tile_mean_workspace_bytes(int B, int N, int D, int F, int c) {
    if (check_mlp_shapes(B, N, D, F, c) != CHIPMUNK_OK) return 0;
    const int64_t units = (int64_t)B * ((N + c - 1) / c);
    if (units > 0x7fffff) return 0;
    return tile_mean_bytes(B, N, D, F, c, tile_mean_pieces((int)units, F));
}

// The column-sparse delta MLP; `deferred`: the activation-cache write-back runs in the second GEMM's launch
// (workspace: delta^T, then the new activations in the same layout).
static int32_t run_mlp_sparse_delta(const uint16_t* x, const uint16_t* w1, const uint16_t* b1, const uint16_t* w2,
                                    const int32_t* idx, const int32_t* counts, uint16_t* a_cache, int64_t a_ld,
                                    uint16_t* o_cache, int B, int N, int D, int F, int c, int k_stride, int act,
                                    void* ws, size_t ws_bytes, void* stream, bool deferred) {
    if (!x || !w1 || !w2 || !idx || !counts || !a_cache || !o_cache) return CHIPMUNK_ERR_NULL;
    int32_t st = check_mlp_shapes(B, N, D, F, c);
    if (st != CHIPMUNK_OK) return st;
    if (k_stride < 0 || k_stride > F || a_ld < N) return CHIPMUNK_ERR_SHAPE;
    if (act != CHIPMUNK_ACT_GELU_ERF && act != CHIPMUNK_ACT_GELU_TANH) return CHIPMUNK_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(a_cache) || !aligned16(o_cache) ||
        !aligned16(idx) || !aligned16(counts) || !aligned16(ws) || (reinterpret_cast<uintptr_t>(b1) & 1u) ||
        (a_ld % 8) != 0)
        return CHIPMUNK_ERR_ALIGN;
    if (k_stride == 0) return CHIPMUNK_OK;
    const size_t delta_bytes = chipmunk_mlp_workspace_bytes(B, N, D, F, c, k_stride);
    const size_t need = deferred ? 2 * delta_bytes : delta_bytes;
    if (!ws || ws_bytes < need) return CHIPMUNK_ERR_WORKSPACE;
    const int NB = (N + c - 1) / c, units = B * NB;
    const int k_pad = round_up(k_stride, kBN);
    hipStream_t s = (hipStream_t)stream;
    uint16_t* act_t = deferred ? (uint16_t*)((char*)ws + delta_bytes) : nullptr;

    Gemm1Params g1;
    g1.x = x; g1.w1 = w1; g1.b1 = b1; g1.idx = idx; g1.counts = counts; g1.a_cache = a_cache;
    g1.delta_t = (uint16_t*)ws; g1.act_t = act_t; g1.out_f32 = nullptr; g1.a_ld = a_ld;
    g1.N = N; g1.NB = NB; g1.D = D; g1.F = F; g1.K = D; g1.ldx = D;
    g1.k_stride = k_stride; g1.k_pad = k_pad; g1.act = act; g1.ksplit = 1;
    st = c == 192 ? launch_gemm1<192, kSparseDelta>(g1, k_pad / kBN, units, s)
                  : launch_gemm1<128, kSparseDelta>(g1, k_pad / kBN, units, s);
    if (st != CHIPMUNK_OK) return st;

    Gemm2Params g2;
    g2.a_t = (const uint16_t*)ws; g2.w2 = w2; g2.bias = nullptr; g2.idx = idx; g2.counts = counts; g2.o = o_cache;
    g2.a_ld = a_ld; g2.N = N; g2.NB = NB; g2.D = D; g2.F = F; g2.k_stride = k_stride; g2.k_pad = k_pad; g2.dense = 0;
    g2.act_t = act_t; g2.a_cache = a_cache;
    return c == 192 ? launch_gemm2<192>(g2, D / kBN, units, s) : launch_gemm2<128>(g2, D / kBN, units, s);
}

extern "C" int32_t chipmunk_mlp_sparse_delta(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                                             const uint16_t* w2, const int32_t* idx, const int32_t* counts,
                                             uint16_t* a_cache, int64_t a_ld, uint16_t* o_cache, int B, int N,
                                             int D, int F, int c, int k_stride, int act, void* ws,
                                             size_t ws_bytes, void* stream) {
    return run_mlp_sparse_delta(x, w1, b1, w2, idx, counts, a_cache, a_ld, o_cache, B, N, D, F, c, k_stride, act, ws,
                                ws_bytes, stream, false);
}

extern "C" size_t chipmunk_mlp_overlapped_workspace_bytes(int B, int N, int D, int F, int c, int k_stride) {
    return 2 * chipmunk_mlp_workspace_bytes(B, N, D, F, c, k_stride);
}

extern "C" int32_t chipmunk_mlp_sparse_delta_overlapped(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                                                        const uint16_t* w2, const int32_t* idx,
                                                        const int32_t* counts, uint16_t* a_cache, int64_t a_ld,
                                                        uint16_t* o_cache, int B, int N, int D, int F, int c,
                                                        int k_stride, int act, void* ws, size_t ws_bytes,
                                                        void* stream) {
    return run_mlp_sparse_delta(x, w1, b1, w2, idx, counts, a_cache, a_ld, o_cache, B, N, D, F, c, k_stride, act, ws,
                                ws_bytes, stream, true);
}

extern "C" int32_t chipmunk_mlp_dense(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                                      const uint16_t* w2, const uint16_t* b2, uint16_t* out, uint16_t* a_cache,
                                      int64_t a_ld, int B, int N, int D, int F, int c, int act, void* stream) {
    if (!x || !w1 || !w2 || !out || !a_cache) return CHIPMUNK_ERR_NULL;
    int32_t st = check_mlp_shapes(B, N, D, F, c);
    if (st != CHIPMUNK_OK) return st;
    if (a_ld < N) return CHIPMUNK_ERR_SHAPE;
    if ((int64_t)F * a_ld * 2 >= (1LL << 32)) return CHIPMUNK_ERR_SHAPE;
    if (act != CHIPMUNK_ACT_GELU_ERF && act != CHIPMUNK_ACT_GELU_TANH) return CHIPMUNK_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(a_cache) || !aligned16(out) ||
        (reinterpret_cast<uintptr_t>(b1) & 1u) || (reinterpret_cast<uintptr_t>(b2) & 7u) || (a_ld % 8) != 0)
        return CHIPMUNK_ERR_ALIGN;
    const int NB = (N + c - 1) / c, units = B * NB;
    hipStream_t s = (hipStream_t)stream;

    Gemm1Params g1;
    g1.x = x; g1.w1 = w1; g1.b1 = b1; g1.idx = nullptr; g1.counts = nullptr; g1.a_cache = a_cache;
    g1.delta_t = nullptr; g1.act_t = nullptr; g1.out_f32 = nullptr; g1.a_ld = a_ld;
    g1.N = N; g1.NB = NB; g1.D = D; g1.F = F; g1.K = D; g1.ldx = D;
    g1.k_stride = F; g1.k_pad = F; g1.act = act; g1.ksplit = 1;
    st = c == 192 ? launch_gemm1<192, kDenseAct>(g1, (F + kBN - 1) / kBN, units, s)
                  : launch_gemm1<128, kDenseAct>(g1, (F + kBN - 1) / kBN, units, s);
    if (st != CHIPMUNK_OK) return st;

    Gemm2Params g2;
    g2.a_t = a_cache; g2.w2 = w2; g2.bias = b2; g2.idx = nullptr; g2.counts = nullptr; g2.o = out;
    g2.a_ld = a_ld; g2.N = N; g2.NB = NB; g2.D = D; g2.F = F; g2.k_stride = F; g2.k_pad = F; g2.dense = 1;
    g2.act_t = nullptr; g2.a_cache = nullptr;
    return c == 192 ? launch_gemm2<192>(g2, D / kBN, units, s) : launch_gemm2<128>(g2, D / kBN, units, s);
}

// chunk means -> scores GEMM (-> sum of the pieces); ws holds tile_mean_bytes(..., pieces) bytes
static int32_t run_tile_mean(const uint16_t* x, const uint16_t* w1, float* T, int B, int N, int D, int F, int c,
                             void* ws, int pieces, hipStream_t s) {
    const int NB = (N + c - 1) / c, units = B * NB;
    hipLaunchKernelGGL(chunk_mean_kernel, dim3((unsigned)(((D / 8 + 63) / 64) * units)), dim3(256), 0, s, x, (uint16_t*)ws,
                       N, NB, D, c);
    if (launch_status() != CHIPMUNK_OK) return CHIPMUNK_ERR_LAUNCH;
    // scores[unit, f] = <[hi | lo](unit), [w1_f | w1_f]>: a plain GEMM with "tokens" = units
    size_t means = ((size_t)units * 2 * D * 2 + 255) / 256 * 256;
    float* partial = pieces > 1 ? (float*)((char*)ws + means) : T;
    Gemm1Params g1;
    g1.x = (const uint16_t*)ws; g1.w1 = w1; g1.b1 = nullptr; g1.idx = nullptr; g1.counts = nullptr;
    g1.a_cache = nullptr; g1.delta_t = nullptr; g1.act_t = nullptr; g1.out_f32 = partial; g1.a_ld = 0;
    g1.N = units; g1.NB = (units + 127) / 128; g1.D = D; g1.F = F; g1.K = 2 * D; g1.ldx = 2 * D;
    g1.k_stride = F; g1.k_pad = F; g1.act = 0; g1.ksplit = pieces;
    int32_t st = launch_gemm1<128, kPlainF32>(g1, (F + kBN - 1) / kBN, g1.NB, s);
    if (st != CHIPMUNK_OK || pieces == 1) return st;
    int64_t n4 = (int64_t)units * F / 4;
    hipLaunchKernelGGL(sum_pieces_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, s, partial, T, n4, pieces);
    return launch_status();
}

extern "C" int32_t chipmunk_mlp_tile_mean_preact(const uint16_t* x, const uint16_t* w1, float* T, int B, int N,
                                                 int D, int F, int c, void* ws, size_t ws_bytes, void* stream) {
    if (!x || !w1 || !T) return CHIPMUNK_ERR_NULL;
    int32_t st = check_mlp_shapes(B, N, D, F, c);
    if (st != CHIPMUNK_OK) return st;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(T) || !aligned16(ws)) return CHIPMUNK_ERR_ALIGN;
    const int64_t units = (int64_t)B * ((N + c - 1) / c);
    if (units > 0x7fffff || units * 2 * D * 2 >= (1LL << 32)) return CHIPMUNK_ERR_SHAPE;
    const int pieces = tile_mean_pieces((int)units, F);
    size_t need = tile_mean_bytes(B, N, D, F, c, pieces);
    if (!ws || need == 0 || ws_bytes < need) return CHIPMUNK_ERR_WORKSPACE;
    return run_tile_mean(x, w1, T, B, N, D, F, c, ws, pieces, (hipStream_t)stream);
}

// ---- the token-merged pre-activation for callers that cannot allocate ---------------------------------------
// Same kernels as chipmunk_mlp_tile_mean_preact; the workspace is a fixed array in device memory that belongs to
// the library.  Each GPU the library runs on holds its own copy at its own address: the address is looked up once
// per device (with that device current) and kept; host code passes that address, never the array's name, to the
// kernels.
namespace chipmunk {

constexpr size_t kStaticScratchBytes = 32u << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) uint8_t scratch[kStaticScratchBytes];

static std::mutex scratch_mutex;
static void* scratch_address[kMaxDevices];   // per device, 0 until looked up

static int32_t scratch_of_current_device(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CHIPMUNK_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_address[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return CHIPMUNK_ERR_LAUNCH;
        scratch_address[dev] = ptr;
    }
    *out = scratch_address[dev];
    return CHIPMUNK_OK;
}

}  // namespace chipmunk

extern "C" size_t chipmunk_mlp_tile_mean_preact_static_capacity(void) { return kStaticScratchBytes; }

extern "C" int32_t chipmunk_mlp_tile_mean_preact_static(const uint16_t* x, const uint16_t* w1, float* T, int B, int N,
                                                        int D, int F, int c, void* stream) {
    if (!x || !w1 || !T) return CHIPMUNK_ERR_NULL;
    int32_t st = check_mlp_shapes(B, N, D, F, c);
    if (st != CHIPMUNK_OK) return st;
    if (!aligned16(x) || !aligned16(w1) || !aligned16(T)) return CHIPMUNK_ERR_ALIGN;
    const int64_t units = (int64_t)B * ((N + c - 1) / c);
    if (units > 0x7fffff || units * 2 * D * 2 >= (1LL << 32)) return CHIPMUNK_ERR_SHAPE;
    // as many pieces of the contraction as the general entry point would use, halved until the chunk means and the
    // pieces' partial results fit the array; with one piece the scores go straight to T
    int pieces = tile_mean_pieces((int)units, F);
    while (pieces > 1 && tile_mean_bytes(B, N, D, F, c, pieces) > kStaticScratchBytes) pieces /= 2;
    const size_t need = tile_mean_bytes(B, N, D, F, c, pieces);
    if (need == 0 || need > kStaticScratchBytes) return CHIPMUNK_ERR_WORKSPACE;   // the chunk means alone do not fit
    void* ws = nullptr;
    st = scratch_of_current_device(&ws);
    if (st != CHIPMUNK_OK) return st;
    // every byte of the array that the kernels read in this call is written by this call first (the chunk means
    // by chunk_mean_kernel, every piece's partial scores by the scores GEMM): nothing has to start at zero
    return run_tile_mean(x, w1, T, B, N, D, F, c, ws, pieces, (hipStream_t)stream);
}
