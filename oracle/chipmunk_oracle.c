/*
 * CPU oracle for the Chipmunk hot path (arXiv 2506.03275): voxel token
 * reorder, per-chunk top-k column selection, column-sparse delta attention,
 * column-sparse delta MLP, and the dense operations that fill their caches.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition of what the
 * GPU library must compute.  Only tests, the smoke check and the CPU-baseline
 * leg of the benchmark may load it; the GPU library never does, and the two
 * share no code.  Floating-point work is done in double on inputs that are
 * given as float (bf16 values widened exactly).  The one exception is the
 * top-k score |cur - prev|, which is a decision taken in float on both sides.
 *
 * Loops are parallelised with OpenMP over independent units only (a batch
 * row, a (batch, head, query chunk), a (batch, token chunk)); inside a unit
 * the arithmetic is written in the order of the paper's definitions with no
 * blocking, fusion or reordering.
 *
 * Every function returns 0, or a negative number for an argument it rejects.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* Voxel reorder (Alg. 1; Sec. 3.2.1 "Reordering tokens ...").
 *
 * Tokens before the reorder: n_prefix tokens, then the T*H*W grid in raster
 * order (t slowest, w fastest), then n_suffix tokens.
 * Alg. 1 is the pattern  (tc vt)(hc vh)(wc vw) -> tc hc wc vt vh vw.
 * Reading for what the listing leaves open: prefix and suffix tokens keep
 * their places; grid positions that lie outside the last full voxel in any
 * dimension follow all full voxels, in raster order.  When vt|T, vh|H, vw|W
 * there is no remainder and this is Alg. 1 exactly.
 *
 * perm[new] = old position, inv_perm[old] = new position.
 */
int oracle_voxel_perm(int n_prefix, int T, int H, int W, int n_suffix,
                      int vt, int vh, int vw, int32_t* perm, int32_t* inv_perm) {
    if (n_prefix < 0 || n_suffix < 0 || T < 1 || H < 1 || W < 1) return -2;
    if (vt < 1 || vh < 1 || vw < 1) return -2;
    int64_t N = (int64_t)n_prefix + (int64_t)T * H * W + n_suffix;
    if (N > INT32_MAX) return -2;
    int tc_n = T / vt, hc_n = H / vh, wc_n = W / vw;
    int64_t pos = 0;
    for (int i = 0; i < n_prefix; i++) perm[pos++] = i;
    for (int tc = 0; tc < tc_n; tc++)
        for (int hc = 0; hc < hc_n; hc++)
            for (int wc = 0; wc < wc_n; wc++)
                for (int dt = 0; dt < vt; dt++)
                    for (int dh = 0; dh < vh; dh++)
                        for (int dw = 0; dw < vw; dw++) {
                            int t = tc * vt + dt, h = hc * vh + dh, w = wc * vw + dw;
                            perm[pos++] = n_prefix + (t * H + h) * W + w;
                        }
    for (int t = 0; t < T; t++)
        for (int h = 0; h < H; h++)
            for (int w = 0; w < W; w++) {
                int in_full = (t < tc_n * vt) && (h < hc_n * vh) && (w < wc_n * vw);
                if (!in_full) perm[pos++] = n_prefix + (t * H + h) * W + w;
            }
    for (int i = 0; i < n_suffix; i++) perm[pos++] = n_prefix + T * H * W + i;
    if (pos != N) return -7;
    if (inv_perm)
        for (int64_t i = 0; i < N; i++) inv_perm[perm[i]] = (int32_t)i;
    return 0;
}

/* Apply the permutation to rows of row_bytes bytes.
 * forward (inverse == 0): dst[b][i]       = src[b][perm[i]]   (voxel_order)
 * inverse (inverse != 0): dst[b][perm[i]] = src[b][i]         (reverse_voxel_order) */
int oracle_reorder_rows(const uint8_t* src, uint8_t* dst, const int32_t* perm,
                        int batch, int N, int row_bytes, int inverse) {
    if (batch < 0 || N < 0 || row_bytes < 1) return -2;
    for (int b = 0; b < batch; b++)
        for (int i = 0; i < N; i++) {
            int64_t from = inverse ? i : perm[i];
            int64_t to = inverse ? perm[i] : i;
            memcpy(dst + ((int64_t)b * N + to) * row_bytes,
                   src + ((int64_t)b * N + from) * row_bytes, (size_t)row_bytes);
        }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Top-k columns (Sec. 3.3.1 "idx = TopK_k(D)"; Sec. 3.3.2 / Alg. 7
 * "idx = TopK(|T - T_m|)").
 *
 * score_j = cur_j, or |cur_j - prev_j| evaluated in float when prev is given.
 * The k columns of largest score are kept; of equal scores the lower column
 * wins; the kept columns are written in ascending order; counts[r] = k.
 * Entries k..k_stride-1 of a row of idx are left as they were.
 * This is the definition written out: sort all columns by (score descending,
 * column ascending), take the first k, sort those by column.
 */
typedef struct { float score; int32_t col; } scored_col;

static int cmp_score_desc(const void* a, const void* b) {
    const scored_col* x = (const scored_col*)a;
    const scored_col* y = (const scored_col*)b;
    if (x->score > y->score) return -1;
    if (x->score < y->score) return 1;
    return (x->col > y->col) - (x->col < y->col);
}
static int cmp_int32(const void* a, const void* b) {
    int32_t x = *(const int32_t*)a, y = *(const int32_t*)b;
    return (x > y) - (x < y);
}

int oracle_topk_cols(const float* cur, const float* prev, int R, int C, int64_t ld,
                     int k, int32_t* idx, int32_t* counts, int k_stride) {
    if (R < 0 || C < 1 || ld < C || k < 0 || k > C || k_stride < k) return -2;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < R; r++) {
        scored_col* s = (scored_col*)malloc(sizeof(scored_col) * (size_t)C);
        if (!s) { err = 1; continue; }
        for (int j = 0; j < C; j++) {
            float x = cur[(int64_t)r * ld + j];
            if (prev) {
                volatile float d = x - prev[(int64_t)r * ld + j]; /* one float subtract */
                x = fabsf(d);
            }
            if (x == 0.0f) x = 0.0f; /* -0 and +0 are the same score */
            s[j].score = x;
            s[j].col = j;
        }
        qsort(s, (size_t)C, sizeof(scored_col), cmp_score_desc);
        int32_t* out = idx + (int64_t)r * k_stride;
        for (int j = 0; j < k; j++) out[j] = s[j].col;
        qsort(out, (size_t)k, sizeof(int32_t), cmp_int32);
        counts[r] = k;
        free(s);
    }
    return err ? -8 : 0;
}

/* ------------------------------------------------------------------------ */
/* Bit-packed column masks (App. B.4 "Bitpacked Sparsity Masks") and the conversion
 * between a mask and the index list of its row (Table 3 "mask to indices").
 * mask is [R, ld_words] 32-bit words; bit (j % 32) of word j / 32 stands for column j.
 *   mask -> indices: the set columns below C in ascending order, at most k_stride of
 *   them; counts[r] = how many were written.
 *   indices -> mask: every bit of the row's words is cleared, then the bit of every
 *   listed column that lies in [0, C) is set. */
int oracle_mask_to_indices(const uint32_t* mask, int64_t ld_words, int R, int C,
                           int32_t* idx, int32_t* counts, int k_stride) {
    if (R < 0 || C < 1 || k_stride < 0 || ld_words < (C + 31) / 32) return -2;
    for (int r = 0; r < R; r++) {
        int n = 0;
        for (int j = 0; j < C; j++) {
            uint32_t word = mask[(int64_t)r * ld_words + j / 32];
            if ((word >> (j % 32)) & 1u) {
                if (n < k_stride) idx[(int64_t)r * k_stride + n] = j;
                n++;
            }
        }
        counts[r] = n < k_stride ? n : k_stride;
    }
    return 0;
}

int oracle_indices_to_mask(const int32_t* idx, const int32_t* counts, int R, int C, int k_stride,
                           uint32_t* mask, int64_t ld_words) {
    if (R < 0 || C < 1 || k_stride < 0 || ld_words < (C + 31) / 32) return -2;
    for (int r = 0; r < R; r++) {
        for (int w = 0; w < (C + 31) / 32; w++) mask[(int64_t)r * ld_words + w] = 0u;
        int n = counts[r] < k_stride ? counts[r] : k_stride;
        for (int j = 0; j < n; j++) {
            int32_t col = idx[(int64_t)r * k_stride + j];
            if (col >= 0 && col < C) mask[(int64_t)r * ld_words + col / 32] |= 1u << (col % 32);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Dense attention and exact column sums (Sec. 3.3.1 "Dense Steps").
 *   P = softmax(scale * Q K^T) row-wise,  O = P V,
 *   D[b,h,i,j] = sum over the rows q of chunk i of P[b,h,q,j].
 * q is [B,H,Nq,E]; k and v are [B,H,Nk,E]; out is [B,H,Nq,E]; colsum (may be
 * NULL) is [B,H,ceil(Nq/c),Nk].  The last chunk may hold fewer than c rows.
 */
int oracle_attn_dense(const float* q, const float* k, const float* v, double* out,
                      double* colsum, int B, int H, int Nq, int Nk, int E, int c,
                      double scale) {
    if (B < 1 || H < 1 || Nq < 1 || Nk < 1 || E < 1 || c < 1) return -2;
    int NB = (Nq + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int64_t bh = u / NB;
        int i = (int)(u % NB);
        const float* kk = k + bh * Nk * E;
        const float* vv = v + bh * Nk * E;
        double* p = (double*)malloc(sizeof(double) * (size_t)Nk);
        if (!p) { err = 1; continue; }
        double* cs = colsum ? colsum + (bh * NB + i) * Nk : NULL;
        if (cs) for (int j = 0; j < Nk; j++) cs[j] = 0.0;
        int r1 = (i + 1) * c < Nq ? (i + 1) * c : Nq;
        for (int r = i * c; r < r1; r++) {
            const float* qr = q + (bh * Nq + r) * E;
            double m = -INFINITY;
            for (int j = 0; j < Nk; j++) {
                double s = 0.0;
                for (int e = 0; e < E; e++) s += (double)qr[e] * (double)kk[(int64_t)j * E + e];
                p[j] = scale * s;
                if (p[j] > m) m = p[j];
            }
            double l = 0.0;
            for (int j = 0; j < Nk; j++) { p[j] = exp(p[j] - m); l += p[j]; }
            for (int j = 0; j < Nk; j++) p[j] /= l;
            double* o = out + (bh * Nq + r) * E;
            for (int e = 0; e < E; e++) o[e] = 0.0;
            for (int j = 0; j < Nk; j++)
                for (int e = 0; e < E; e++) o[e] += p[j] * (double)vv[(int64_t)j * E + e];
            if (cs) for (int j = 0; j < Nk; j++) cs[j] += p[j];
        }
        free(p);
    }
    return err ? -8 : 0;
}

/* Row statistics of dense attention: m[b,h,n] = max_j scale*<Q_n,K_j> and
 * l[b,h,n] = sum_j exp(scale*<Q_n,K_j> - m[b,h,n]), the softmax normalisers that
 * Alg. 4 carries from one step to the next (prev_m, prev_l).
 */
int oracle_attn_row_stats(const float* q, const float* k, double* m_out, double* l_out,
                          int B, int H, int Nq, int Nk, int E, double scale) {
    if (B < 1 || H < 1 || Nq < 1 || Nk < 1 || E < 1) return -2;
    int64_t rows = (int64_t)B * H * Nq;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < rows; n++) {
        int64_t bh = n / Nq;
        const float* qr = q + n * E;
        const float* kk = k + bh * Nk * E;
        double m = -INFINITY;
        for (int j = 0; j < Nk; j++) {
            double s = 0.0;
            for (int e = 0; e < E; e++) s += (double)qr[e] * (double)kk[(int64_t)j * E + e];
            s *= scale;
            if (s > m) m = s;
        }
        double l = 0.0;
        for (int j = 0; j < Nk; j++) {
            double s = 0.0;
            for (int e = 0; e < E; e++) s += (double)qr[e] * (double)kk[(int64_t)j * E + e];
            l += exp(scale * s - m);
        }
        m_out[n] = m;
        l_out[n] = l;
    }
    return 0;
}

/* Column sums with given (stale) normalisers (Alg. 4; App. B.2):
 *   p_approx[n,j] = exp(scale*<Q_n,K_j> - prev_m[n]) / prev_l[n],
 *   cs[b,h,i,j]   = sum over the rows n of chunk i of p_approx[n,j].
 * prev_m, prev_l are [B,H,Nq]; cs is [B,H,ceil(Nq/c),Nk].
 */
int oracle_attn_colsum_stale(const float* q, const float* k, const double* prev_m,
                             const double* prev_l, double* cs, int B, int H, int Nq, int Nk,
                             int E, int c, double scale) {
    if (B < 1 || H < 1 || Nq < 1 || Nk < 1 || E < 1 || c < 1) return -2;
    int NB = (Nq + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int64_t bh = u / NB;
        int i = (int)(u % NB);
        const float* kk = k + bh * Nk * E;
        double* row = cs + u * Nk;
        for (int j = 0; j < Nk; j++) row[j] = 0.0;
        int r1 = (i + 1) * c < Nq ? (i + 1) * c : Nq;
        for (int r = i * c; r < r1; r++) {
            const float* qr = q + (bh * Nq + r) * E;
            double m = prev_m[bh * Nq + r], l = prev_l[bh * Nq + r];
            for (int j = 0; j < Nk; j++) {
                double s = 0.0;
                for (int e = 0; e < E; e++) s += (double)qr[e] * (double)kk[(int64_t)j * E + e];
                row[j] += exp(scale * s - m) / l;
            }
        }
    }
    return 0;
}

/* Column-sparse delta attention (Sec. 3.3.1 "Sparse Delta Steps"; Alg. 3).
 * For chunk i of (b,h) with S = idx[b,h,i,0:counts[b,h,i]] and each of its
 * rows q:
 *   s_j = scale * <Q_q, K_j>  (j in S),   p = softmax over S only,
 *   out_q = base_q + o_scale * sum_{j in S} p_j V_j.
 * counts == 0 leaves out_q = base_q.  A column listed twice counts twice.
 * q, base, out are [B,H,Nq,E]; k, v are [B,H,Nk,E]; idx is
 * [B,H,ceil(Nq/c),k_stride]; counts is [B,H,ceil(Nq/c)].
 */
int oracle_attn_sparse_delta(const float* q, const float* k, const float* v,
                             const int32_t* idx, const int32_t* counts,
                             const double* base, double* out, int B, int H, int Nq,
                             int Nk, int E, int c, int k_stride, double scale,
                             double o_scale) {
    if (B < 1 || H < 1 || Nq < 1 || Nk < 1 || E < 1 || c < 1 || k_stride < 0) return -2;
    int NB = (Nq + c - 1) / c;
    int64_t units = (int64_t)B * H * NB;
    for (int64_t u = 0; u < units; u++) {
        if (counts[u] < 0 || counts[u] > k_stride) return -2;
        for (int t = 0; t < counts[u]; t++) {
            int32_t j = idx[u * k_stride + t];
            if (j < 0 || j >= Nk) return -2;
        }
    }
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int64_t bh = u / NB;
        int i = (int)(u % NB);
        const float* kk = k + bh * Nk * E;
        const float* vv = v + bh * Nk * E;
        const int32_t* S = idx + u * k_stride;
        int cnt = counts[u];
        double* p = (double*)malloc(sizeof(double) * (size_t)(cnt > 0 ? cnt : 1));
        if (!p) { err = 1; continue; }
        int r1 = (i + 1) * c < Nq ? (i + 1) * c : Nq;
        for (int r = i * c; r < r1; r++) {
            const float* qr = q + (bh * Nq + r) * E;
            const double* br = base + (bh * Nq + r) * E;
            double* o = out + (bh * Nq + r) * E;
            if (cnt == 0) {
                for (int e = 0; e < E; e++) o[e] = br[e];
                continue;
            }
            double m = -INFINITY;
            for (int t = 0; t < cnt; t++) {
                const float* kj = kk + (int64_t)S[t] * E;
                double s = 0.0;
                for (int e = 0; e < E; e++) s += (double)qr[e] * (double)kj[e];
                p[t] = scale * s;
                if (p[t] > m) m = p[t];
            }
            double l = 0.0;
            for (int t = 0; t < cnt; t++) { p[t] = exp(p[t] - m); l += p[t]; }
            for (int e = 0; e < E; e++) {
                double d = 0.0;
                for (int t = 0; t < cnt; t++) d += (p[t] / l) * (double)vv[(int64_t)S[t] * E + e];
                o[e] = br[e] + o_scale * d;
            }
        }
        free(p);
    }
    return err ? -8 : 0;
}

/* ------------------------------------------------------------------------ */
/* Activation: 0 = GELU with erf, 1 = GELU with the tanh approximation. */
static double act_fn(double x, int act) {
    if (act == 0) return 0.5 * x * (1.0 + erf(x / sqrt(2.0)));
    const double pi = 3.14159265358979323846;
    double u = sqrt(2.0 / pi) * (x + 0.044715 * x * x * x);
    return 0.5 * x * (1.0 + tanh(u));
}

/* Dense MLP and the three caches of a dense step (Sec. 3.3.2 "Dense steps";
 * Alg. 5):  A = act(X W1^T + b1),  O = A W2 + b2,
 *   a_cache[b,f,n] = A[b,n,f]   (neuron-major, leading dimension a_ld >= N),
 *   T_m[b,i,f]     = mean over the rows n of chunk i of (X W1^T)[b,n,f]
 *                    (no bias: it would cancel in |T - T_m|).
 * x [B,N,D]; w1, w2 [F,D]; b1 [F] or NULL; b2 [D] or NULL; out [B,N,D];
 * a_cache and T_m may be NULL.
 */
int oracle_mlp_dense(const float* x, const float* w1, const float* b1, const float* w2,
                     const float* b2, double* out, double* a_cache, int64_t a_ld,
                     double* T_m, int B, int N, int D, int F, int c, int act) {
    if (B < 1 || N < 1 || D < 1 || F < 1 || c < 1 || (act != 0 && act != 1)) return -2;
    if (a_cache && a_ld < N) return -2;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * NB;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int b = (int)(u / NB), i = (int)(u % NB);
        int r1 = (i + 1) * c < N ? (i + 1) * c : N;
        int rows = r1 - i * c;
        double* a = (double*)malloc(sizeof(double) * (size_t)F);
        if (!a) { err = 1; continue; }
        if (T_m) for (int f = 0; f < F; f++) T_m[u * F + f] = 0.0;
        for (int n = i * c; n < r1; n++) {
            const float* xr = x + ((int64_t)b * N + n) * D;
            for (int f = 0; f < F; f++) {
                double pre = 0.0;
                for (int d = 0; d < D; d++) pre += (double)xr[d] * (double)w1[(int64_t)f * D + d];
                if (T_m) T_m[u * F + f] += pre / rows;
                if (b1) pre += (double)b1[f];
                a[f] = act_fn(pre, act);
                if (a_cache) a_cache[((int64_t)b * F + f) * a_ld + n] = a[f];
            }
            double* o = out + ((int64_t)b * N + n) * D;
            for (int d = 0; d < D; d++) o[d] = b2 ? (double)b2[d] : 0.0;
            for (int f = 0; f < F; f++)
                for (int d = 0; d < D; d++) o[d] += a[f] * (double)w2[(int64_t)f * D + d];
        }
        free(a);
    }
    return err ? -8 : 0;
}

/* Token-merged pre-activation of a sparse step (Alg. 7):
 *   T[b,i,:] = (mean over the rows of chunk i of X[b]) @ W1^T, no bias. */
int oracle_mlp_tile_scores(const float* x, const float* w1, double* T, int B, int N,
                           int D, int F, int c) {
    if (B < 1 || N < 1 || D < 1 || F < 1 || c < 1) return -2;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * NB;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int b = (int)(u / NB), i = (int)(u % NB);
        int r1 = (i + 1) * c < N ? (i + 1) * c : N;
        int rows = r1 - i * c;
        double* xm = (double*)malloc(sizeof(double) * (size_t)D);
        if (!xm) { err = 1; continue; }
        for (int d = 0; d < D; d++) {
            double s = 0.0;
            for (int n = i * c; n < r1; n++) s += (double)x[((int64_t)b * N + n) * D + d];
            xm[d] = s / rows;
        }
        for (int f = 0; f < F; f++) {
            double t = 0.0;
            for (int d = 0; d < D; d++) t += xm[d] * (double)w1[(int64_t)f * D + d];
            T[u * F + f] = t;
        }
        free(xm);
    }
    return err ? -8 : 0;
}

/* Column-sparse delta MLP (Sec. 3.3.2 "Sparse Delta Steps"; App. B.3.1;
 * Alg. 6).  For chunk i of batch b with S = idx[b,i,0:counts[b,i]], each of
 * its rows n and each f in S:
 *   a = act(<X_n, W1_f> + b1_f),  delta = a - a_cache[b,f,n],  a_cache[b,f,n] = a,
 * then  o_cache[b,n,:] += sum_{f in S} delta_{n,f} W2_f.
 * b2 is not added again: it is already inside o_cache.
 */
int oracle_mlp_sparse_delta(const float* x, const float* w1, const float* b1,
                            const float* w2, const int32_t* idx, const int32_t* counts,
                            double* a_cache, int64_t a_ld, double* o_cache, int B, int N,
                            int D, int F, int c, int k_stride, int act) {
    if (B < 1 || N < 1 || D < 1 || F < 1 || c < 1 || k_stride < 0) return -2;
    if (a_ld < N || (act != 0 && act != 1)) return -2;
    int NB = (N + c - 1) / c;
    int64_t units = (int64_t)B * NB;
    for (int64_t u = 0; u < units; u++) {
        if (counts[u] < 0 || counts[u] > k_stride) return -2;
        for (int t = 0; t < counts[u]; t++) {
            int32_t f = idx[u * k_stride + t];
            if (f < 0 || f >= F) return -2;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; u++) {
        int b = (int)(u / NB), i = (int)(u % NB);
        int r1 = (i + 1) * c < N ? (i + 1) * c : N;
        const int32_t* S = idx + u * k_stride;
        int cnt = counts[u];
        for (int n = i * c; n < r1; n++) {
            const float* xr = x + ((int64_t)b * N + n) * D;
            double* o = o_cache + ((int64_t)b * N + n) * D;
            for (int t = 0; t < cnt; t++) {
                int f = S[t];
                double pre = 0.0;
                for (int d = 0; d < D; d++) pre += (double)xr[d] * (double)w1[(int64_t)f * D + d];
                if (b1) pre += (double)b1[f];
                double a = act_fn(pre, act);
                double* slot = a_cache + ((int64_t)b * F + f) * a_ld + n;
                double delta = a - *slot;
                *slot = a;
                for (int d = 0; d < D; d++) o[d] += delta * (double)w2[(int64_t)f * D + d];
            }
        }
    }
    return 0;
}
