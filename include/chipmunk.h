/*
 * chipmunk.h - C ABI of the MI355X (gfx950) implementation of the Chipmunk hot
 * path (arXiv 2506.03275): dynamic column-sparse delta recompute for
 * Diffusion-Transformer attention and MLP layers.
 *
 * Conventions for every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or synchronises; a call enqueues its kernels on
 *     `stream` (a hipStream_t passed as void*; NULL = the default stream) and
 *     returns at once.
 *   - Tensors are dense and row-major in the layouts stated per call.  bf16
 *     values are passed as raw uint16_t.  Pointers to bf16/fp32/int32 tensors
 *     must be 16-byte aligned.
 *   - Return value: CHIPMUNK_OK, or a negative code; on any error nothing was
 *     launched.  chipmunk_status_string() gives a text for a code.
 *   - Index contents (range, duplicates) are preconditions that are not
 *     reported: every idx entry below its row's count must lie in [0, C) and
 *     every count in [0, k_stride].  The kernels clamp both into range, so a
 *     bad entry gives a wrong result for its chunk, not an access outside the
 *     tensors.
 *   - "chunk" = c consecutive tokens that share one set of selected columns
 *     (the [C,1] column sparsity of Sec. 3.2.1); the last chunk of a sequence
 *     may hold fewer than c tokens.  NB = ceil(N / c).
 */
#ifndef CHIPMUNK_H
#define CHIPMUNK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHIPMUNK_OK                0
#define CHIPMUNK_ERR_NULL         -1  /* a required pointer is NULL */
#define CHIPMUNK_ERR_SHAPE        -2  /* a size is out of range (<= 0, k > C, k_stride < k, ...) */
#define CHIPMUNK_ERR_ALIGN        -3  /* a pointer or leading dimension breaks the alignment rule */
#define CHIPMUNK_ERR_UNSUPPORTED  -4  /* E not in {64,128}, c not in {128,192}, D % 128 or F % 64 != 0, unknown act */
#define CHIPMUNK_ERR_WORKSPACE    -5  /* workspace missing or too small */
#define CHIPMUNK_ERR_LAUNCH       -6  /* the HIP runtime refused a launch */

#define CHIPMUNK_ACT_GELU_ERF   0
#define CHIPMUNK_ACT_GELU_TANH  1

const char* chipmunk_status_string(int32_t status);

/* Voxel token reorder and its inverse (Alg. 1; Sec. 3.2.1).
 * A sequence holds n_prefix tokens, a T*H*W grid in raster order (t slowest,
 * w fastest) and n_suffix tokens: N = n_prefix + T*H*W + n_suffix.  After the
 * reorder every full (vt,vh,vw) voxel occupies vt*vh*vw consecutive positions,
 * voxels in (tc,hc,wc) order, tokens inside a voxel in (dt,dh,dw) order; grid
 * positions outside the last full voxel of any dimension follow in raster
 * order; prefix and suffix tokens keep their places.
 *   inverse == 0:  dst[b][i]       = src[b][perm[i]]
 *   inverse != 0:  dst[b][perm[i]] = src[b][i]
 * src, dst: [batch, N, row_bytes] bytes, must not overlap; both NULL = only
 * write the permutation.  perm, inv_perm: [N] int32, each may be NULL;
 * perm[new] = old, inv_perm[old] = new.  row_bytes must be a multiple of 4;
 * rows that are multiples of 16 bytes with 16-byte aligned src/dst move as
 * 128-bit words. */
int32_t chipmunk_voxel_reorder(const void* src, void* dst, int32_t* perm, int32_t* inv_perm,
                               int batch, int n_prefix, int T, int H, int W, int n_suffix,
                               int vt, int vh, int vw, int row_bytes, int inverse, void* stream);

/* Per-row top-k column selection (Sec. 3.3.1 idx = TopK_k(D); Sec. 3.3.2 and
 * Alg. 7 idx = TopK(|T - T_m|)).
 * cur, prev: [R, ld] fp32 with C used columns (ld >= C, ld % 4 == 0); prev may
 * be NULL.  score_j = cur_j, or |cur_j - prev_j| in fp32.  The k columns with
 * the largest score are kept; of equal scores the lower column wins; -0 = +0;
 * NaN scores are a precondition violation.  idx: [R, k_stride] int32 receives
 * the kept columns in ascending order in its first k entries (the rest is left
 * untouched); counts: [R] receives k.  The call is exact, never approximate. */
int32_t chipmunk_topk_cols(const float* cur, const float* prev, int R, int C, int64_t ld, int k,
                           int32_t* idx, int32_t* counts, int k_stride, void* stream);

/* Bit-packed column masks and their conversion to index lists (App. B.4 "Bitpacked Sparsity Masks": a layer's
 * pattern is cached as one bit per (chunk, column), an eighth of a byte mask; Table 3 "mask to indices conversion":
 * one kernel turns it into the lists the delta kernels walk).  mask: [R, ld_words] uint32, ld_words >= ceil(C/32);
 * bit (j % 32) of word j / 32 of row r is set when column j of row r is selected; bits at or beyond C are ignored
 * on input and written as zero.
 *   chipmunk_mask_to_indices: idx[r, 0:counts[r]] = the selected columns of row r in ascending order, counts[r] =
 *     their number: rows may select different numbers of columns.  A row with more than k_stride selected
 *     columns keeps the first k_stride and reports counts[r] = k_stride.  Entries at or beyond counts[r] are left
 *     untouched.  idx: [R, k_stride] int32; counts: [R] int32.
 *   chipmunk_indices_to_mask: the inverse; row r of mask receives exactly the columns idx[r, 0:counts[r]] that lie
 *     in [0, C) (a column listed twice sets its bit once).  C <= 2^20.
 * Both are exact.  One workgroup per row. */
int32_t chipmunk_mask_to_indices(const uint32_t* mask, int64_t ld_words, int R, int C,
                                 int32_t* idx, int32_t* counts, int k_stride, void* stream);
int32_t chipmunk_indices_to_mask(const int32_t* idx, const int32_t* counts, int R, int C, int k_stride,
                                 uint32_t* mask, int64_t ld_words, void* stream);

/* Column-sparse delta attention (Sec. 3.3.1 "Sparse Delta Steps"; Alg. 3).
 * For chunk i of (b,h) with S = idx[b,h,i,0:counts[b,h,i]] and each row n of it:
 *   out[n] = base[n] + o_scale * softmax_{j in S}(softmax_scale * <q[n],k[j]>) v[j]
 * The softmax runs over the selected columns only, in fp32, with bf16 MFMA
 * products accumulated in fp32.  counts == 0 gives out = base.  o_scale = +1
 * is a sparse step on the cache; o_scale = -1 with base = dense output builds
 * the cache O_cache of a dense step (Alg. 2).
 * q, k, v, base, out: [B,H,N,E] bf16; out may alias base.  idx: [B,H,NB,k_stride]
 * int32; counts: [B,H,NB] int32, each in [0, k_stride].  idx == NULL and
 * counts == NULL selects every column 0..N-1 (dense attention on the same
 * kernel; base may then be NULL, meaning zero).
 * E in {64,128}; c in {128,192}; N*E must stay below 2^31 elements (32-bit byte
 * offsets of K/V rows inside one head; the same limit holds for every attention
 * entry point below).  softmax_scale must be positive and finite, o_scale finite
 * (both are checked on their bit patterns: a NaN is rejected, nothing is launched). */
int32_t chipmunk_attn_sparse_delta(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                   const int32_t* idx, const int32_t* counts,
                                   const uint16_t* base, uint16_t* out,
                                   int B, int H, int N, int E, int c, int k_stride,
                                   float softmax_scale, float o_scale, void* stream);

/* Block-sparse delta attention: the [c, 128] block pattern that Table 2 sets beside the [c, 1] columns
 * (Sec. 3.2.1).  blocks[b,h,i,0:block_counts[b,h,i]] names blocks of CHIPMUNK_ATTN_BLOCK_COLUMNS consecutive
 * key columns (block j = columns 128 j .. 128 j + 127, cut at N); the result is that of
 * chipmunk_attn_sparse_delta on the list of all columns of those blocks:
 *   out[n] = base[n] + o_scale * softmax_{j in the selected blocks}(softmax_scale * <q[n],k[j]>) v[j].
 * The kernel fetches each block's K and V rows as contiguous runs, with no per-column index.  A block listed
 * twice counts twice (the list is taken as given); every entry below its row's count must lie in
 * [0, ceil(N/128)).  blocks: [B,H,NB,kb_stride] int32; block_counts: [B,H,NB] int32, each in [0, kb_stride];
 * block_counts == 0 gives out = base.  Other arguments and limits as for chipmunk_attn_sparse_delta. */
#define CHIPMUNK_ATTN_BLOCK_COLUMNS 128
int32_t chipmunk_attn_block_sparse_delta(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                         const int32_t* blocks, const int32_t* block_counts,
                                         const uint16_t* base, uint16_t* out,
                                         int B, int H, int N, int E, int c, int kb_stride,
                                         float softmax_scale, float o_scale, void* stream);

/* Workspace bytes of chipmunk_attn_dense when column sums are requested (0 on bad arguments). */
size_t chipmunk_attn_dense_workspace_bytes(int B, int H, int N);

/* Dense attention with exact column sums (Sec. 3.3.1 "Dense Steps"):
 *   out = softmax(softmax_scale * q k^T) v,
 *   colsum[b,h,i,j] = sum over the rows n of chunk i of P[b,h,n,j]   (the tensor D).
 * out: [B,H,N,E] bf16; colsum: [B,H,NB,ld_colsum] fp32 (ld_colsum >= N, multiple
 * of 4) or NULL.  Normalisers are those of the current step (exact sums, not
 * the stale-constant approximation of App. B.2): a first pass writes each row's
 * softmax statistics into ws, a second pass recomputes the scores and sums the
 * normalised probabilities per chunk.  ws (chipmunk_attn_dense_workspace_bytes)
 * is needed only when colsum != NULL.  Afterwards it holds those statistics as
 * two fp32 arrays [B,H,N]: m, the reference each row's exponentials were taken
 * against (in units of the scaled scores; within 2^8 of the row maximum, not
 * necessarily equal to it), then l = sum_j exp(score_j - m): the pair a later
 * step can hand to chipmunk_attn_colsum_stale as (prev_m, prev_l). */
int32_t chipmunk_attn_dense(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                            uint16_t* out, float* colsum, int64_t ld_colsum,
                            int B, int H, int N, int E, int c, float softmax_scale,
                            void* ws, size_t ws_bytes, void* stream);

/* Column sums with given normalisers (Alg. 4; App. B.2: the normalisers of the
 * previous diffusion step stand in for the current ones):
 *   colsum[b,h,i,j] = sum over the rows n of chunk i of
 *                     exp(softmax_scale * <q[n],k[j]> - prev_m[n]) / prev_l[n].
 * With the statistics of the same q, k (as left in the workspace of
 * chipmunk_attn_dense) these are the exact column sums D; with statistics of
 * an earlier step they are the paper's approximation, meant only to rank
 * columns.  q, k: [B,H,N,E] bf16; prev_m, prev_l: [B,H,N] fp32; colsum:
 * [B,H,NB,ld_colsum] fp32 (ld_colsum >= N, multiple of 4; columns N..ld-1 are
 * left untouched).  The sums are meant for normalisers that are close to the
 * current ones; they are exact fp32 evaluations of the formula while every
 * weight exp(score - prev_m) / prev_l stays below 2^126.  A weight beyond that
 * makes its column's sum +inf here (like the formula in fp32).
 * E in {64,128}; c in {128,192}. */
int32_t chipmunk_attn_colsum_stale(const uint16_t* q, const uint16_t* k, const float* prev_m,
                                   const float* prev_l, float* colsum, int64_t ld_colsum,
                                   int B, int H, int N, int E, int c, float softmax_scale, void* stream);

/* Dense attention and the column sums with given normalisers in one pass (Alg. 4):
 *   out = softmax(softmax_scale * q k^T) v            with this step's own normalisers,
 *   colsum[b,h,i,j] = sum over the rows n of chunk i of
 *                     exp(softmax_scale * <q[n],k[j]> - prev_m[n]) / prev_l[n]
 * from the same score tiles (no second pass over q k^T and no workspace).
 * new_m, new_l: [B,H,N] fp32 or both NULL; they receive this step's statistics
 * in the form chipmunk_attn_dense leaves them, for the next step's prev_m,
 * prev_l.  new_m == prev_m and new_l == prev_l (update in place) is allowed:
 * the workgroup of a chunk reads the old values of its own rows, and only
 * those, before it writes the new ones; any other overlap is not.  Other
 * arguments as for chipmunk_attn_colsum_stale and chipmunk_attn_dense.
 * Range: this kernel forms a weight as (probability against the running
 * softmax reference) x (one factor per query), and caps that factor at 2^126.
 * While the largest weight exp(score - prev_m) / prev_l of every query row
 * stays below 2^118 the sums agree with chipmunk_attn_colsum_stale; beyond
 * that (normalisers more than about 80 below a row's current maximum) the
 * row's contributions are scaled down together: a column's sum is then a large
 * finite number or +inf, never NaN, and the two entry points may order such
 * columns differently. */
int32_t chipmunk_attn_dense_colsum_stale(const uint16_t* q, const uint16_t* k, const uint16_t* v,
                                         uint16_t* out, const float* prev_m, const float* prev_l,
                                         float* colsum, int64_t ld_colsum, float* new_m, float* new_l,
                                         int B, int H, int N, int E, int c, float softmax_scale,
                                         void* stream);

/* Workspace bytes of chipmunk_mlp_tile_mean_preact (0 on bad arguments). */
size_t chipmunk_mlp_tile_mean_workspace_bytes(int B, int N, int D, int F, int c);

/* Token-merged pre-activation (Alg. 7; T_m of Sec. 3.3.2):
 *   T[b,i,:] = (mean over the rows of chunk i of x[b]) @ w1^T, no bias.
 * x: [B,N,D] bf16; w1: [F,D] bf16; T: [B,NB,F] fp32.  The chunk mean is formed
 * in fp32 and fed to the bf16 MFMA as a sum of two bf16 numbers (high and low
 * part), so T carries about 16 bits of the mean.  D multiple of 128, F of 64.
 * ws: chipmunk_mlp_tile_mean_workspace_bytes(); contents undefined afterwards. */
int32_t chipmunk_mlp_tile_mean_preact(const uint16_t* x, const uint16_t* w1, float* T,
                                      int B, int N, int D, int F, int c,
                                      void* ws, size_t ws_bytes, void* stream);

/* chipmunk_mlp_tile_mean_preact for callers that cannot allocate device memory and so have no workspace to hand
 * in: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and the same result up to the summation order of the contraction's pieces; the workspace is a fixed
 * array of chipmunk_mlp_tile_mean_preact_static_capacity() bytes (32 MiB) in device memory that the library holds
 * on every GPU it runs on until the process ends.  The call allocates and frees nothing.  Problems whose chunk
 * means alone (B * NB * 2 * D bf16 values) exceed the array are rejected with CHIPMUNK_ERR_WORKSPACE and nothing is
 * launched; below that limit the contraction is cut into fewer pieces where the general entry point's workspace
 * would not fit.  All calls on one GPU share that GPU's array: calls that may overlap on one GPU (different
 * streams, or different host threads) race and must be ordered by the caller; nothing in the array has to be
 * cleared between calls.  The first call on a device looks the array's address up (no allocation either); make
 * that call outside stream capture. */
size_t chipmunk_mlp_tile_mean_preact_static_capacity(void);
int32_t chipmunk_mlp_tile_mean_preact_static(const uint16_t* x, const uint16_t* w1, float* T,
                                             int B, int N, int D, int F, int c, void* stream);

/* Workspace bytes of chipmunk_mlp_sparse_delta (0 on bad arguments). */
size_t chipmunk_mlp_workspace_bytes(int B, int N, int D, int F, int c, int k_stride);

/* Column-sparse delta MLP (Sec. 3.3.2 "Sparse Delta Steps"; App. B.3.1; Alg. 6).
 * For chunk i of batch b with S = idx[b,i,0:counts[b,i]], each row n and f in S:
 *   a = act(<x[n], w1[f]> + b1[f]);  delta = a - a_cache[b,f,n];  a_cache[b,f,n] = a
 *   o_cache[b,n,:] += sum_{f in S} delta * w2[f,:]
 * a is rounded to bf16 once; that value is stored and used for delta, so that
 * o_cache = a_cache^T w2 + b2 is preserved up to rounding.  b2 is not added.
 * x: [B,N,D] bf16; w1, w2: [F,D] bf16; b1: [F] bf16 or NULL; idx: [B,NB,k_stride]
 * int32 with distinct entries per row; counts: [B,NB]; a_cache: [B,F,a_ld] bf16,
 * in/out (a_ld >= N, a_ld % 8 == 0); o_cache: [B,N,D] bf16, in/out.
 * ws: workspace of chipmunk_mlp_workspace_bytes(), contents undefined after.
 * D multiple of 128, F multiple of 64; c in {128,192}; act as CHIPMUNK_ACT_*.
 * N*D and F*D must stay below 2^31 elements (32-bit byte offsets inside one
 * batch row block and inside the weights). */
int32_t chipmunk_mlp_sparse_delta(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                                  const uint16_t* w2, const int32_t* idx, const int32_t* counts,
                                  uint16_t* a_cache, int64_t a_ld, uint16_t* o_cache,
                                  int B, int N, int D, int F, int c, int k_stride, int act,
                                  void* ws, size_t ws_bytes, void* stream);

/* The same column-sparse delta MLP with the activation-cache write-back taken out of the first GEMM's epilogue and
 * run inside the second GEMM's launch (App. B.3.3: the memory-bound scatter of the cache updates is overlapped
 * with the compute-bound second GEMM on compute units that its last round of tiles leaves idle).  The first GEMM
 * leaves the new activations in the workspace in the layout of the deltas; the second launch carries one extra
 * workgroup per chunk, with the highest ids, that copies them into a_cache.  Same arguments, and bit for bit the
 * same a_cache and o_cache as chipmunk_mlp_sparse_delta.  ws: chipmunk_mlp_overlapped_workspace_bytes() (twice
 * that of chipmunk_mlp_sparse_delta). */
size_t chipmunk_mlp_overlapped_workspace_bytes(int B, int N, int D, int F, int c, int k_stride);
int32_t chipmunk_mlp_sparse_delta_overlapped(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                                             const uint16_t* w2, const int32_t* idx, const int32_t* counts,
                                             uint16_t* a_cache, int64_t a_ld, uint16_t* o_cache,
                                             int B, int N, int D, int F, int c, int k_stride, int act,
                                             void* ws, size_t ws_bytes, void* stream);

/* Dense MLP of a dense step (Sec. 3.3.2 "Dense steps"; Alg. 5):
 *   a = act(x w1^T + b1) -> a_cache[b,f,n] (bf16, neuron-major);  out = a w2 + b2.
 * out: [B,N,D] bf16; b2: [D] bf16 or NULL; a_cache: [B,F,a_ld] bf16, written
 * (required: the second GEMM reads it).  T_m is produced by
 * chipmunk_mlp_tile_mean_preact on the same x. */
int32_t chipmunk_mlp_dense(const uint16_t* x, const uint16_t* w1, const uint16_t* b1,
                           const uint16_t* w2, const uint16_t* b2, uint16_t* out,
                           uint16_t* a_cache, int64_t a_ld,
                           int B, int N, int D, int F, int c, int act, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CHIPMUNK_H */
