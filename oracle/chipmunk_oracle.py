"""numpy front end of the C oracle (``chipmunk_oracle.c``).  Test infrastructure.

Argument marshalling only: every function checks dtypes and shapes, hands
contiguous host arrays to the C routine of the same name and returns new
arrays (or updates the caches it is given, in place, where the method does).
Floating-point inputs are float32 arrays holding bf16 values widened exactly;
floating-point results are float64.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "chipmunk_oracle.c")
_LIB = os.path.join(_HERE, "libchipmunk_oracle.so")
_lib = None

_i32 = ctypes.c_int32
_i64 = ctypes.c_int64
_f64 = ctypes.c_double
_ptr = ctypes.c_void_p


def build(force=False):
    """Compile the C oracle with gcc (plain -O2, OpenMP, no fast-math, no FMA contraction)."""
    global _lib
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared", "-std=c11",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_num_threads.restype = ctypes.c_int
        for name, args in {
            "oracle_voxel_perm": [_i32] * 8 + [_ptr, _ptr],
            "oracle_reorder_rows": [_ptr, _ptr, _ptr, _i32, _i32, _i32, _i32],
            "oracle_topk_cols": [_ptr, _ptr, _i32, _i32, _i64, _i32, _ptr, _ptr, _i32],
            "oracle_mask_to_indices": [_ptr, _i64, _i32, _i32, _ptr, _ptr, _i32],
            "oracle_indices_to_mask": [_ptr, _ptr, _i32, _i32, _i32, _ptr, _i64],
            "oracle_attn_dense": [_ptr] * 5 + [_i32] * 6 + [_f64],
            "oracle_attn_sparse_delta": [_ptr] * 7 + [_i32] * 7 + [_f64, _f64],
            "oracle_attn_row_stats": [_ptr] * 4 + [_i32] * 5 + [_f64],
            "oracle_attn_colsum_stale": [_ptr] * 5 + [_i32] * 6 + [_f64],
            "oracle_mlp_dense": [_ptr] * 7 + [_i64, _ptr] + [_i32] * 6,
            "oracle_mlp_tile_scores": [_ptr] * 3 + [_i32] * 5,
            "oracle_mlp_sparse_delta": [_ptr] * 7 + [_i64, _ptr] + [_i32] * 7,
        }.items():
            fn = getattr(lib, name)
            fn.argtypes = args
            fn.restype = ctypes.c_int
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(_ptr)


def _arr(a, dtype, shape=None, name="array"):
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need a C-contiguous numpy array of {np.dtype(dtype)}")
    if shape is not None and tuple(a.shape) != tuple(shape):
        raise ValueError(f"{name}: shape {a.shape}, expected {tuple(shape)}")
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"{what} rejected its arguments (code {rc})")


def num_threads():
    return int(_load().oracle_num_threads())


def voxel_perm(n_prefix, T, H, W, n_suffix, vt, vh, vw):
    """(perm, inv_perm): perm[new] = old, inv_perm[old] = new.  Alg. 1."""
    N = n_prefix + T * H * W + n_suffix
    perm = np.empty(N, np.int32)
    inv = np.empty(N, np.int32)
    _check(_load().oracle_voxel_perm(n_prefix, T, H, W, n_suffix, vt, vh, vw, _p(perm), _p(inv)),
           "oracle_voxel_perm")
    return perm, inv


def reorder_rows(src, perm, inverse=False):
    """src [batch, N, ...] of any dtype -> reordered copy.  Alg. 1."""
    src = np.ascontiguousarray(src)
    batch, N = src.shape[0], src.shape[1]
    row_bytes = src.dtype.itemsize * int(np.prod(src.shape[2:], dtype=np.int64))
    _arr(perm, np.int32, (N,), "perm")
    dst = np.empty_like(src)
    _check(_load().oracle_reorder_rows(_p(src), _p(dst), _p(perm), batch, N, row_bytes, int(bool(inverse))),
           "oracle_reorder_rows")
    return dst


def topk_cols(cur, prev, k, k_stride=None, idx_fill=-1):
    """cur, prev [R, C] float32 (prev may be None) -> (idx [R, k_stride] int32, counts [R] int32)."""
    _arr(cur, np.float32, None, "cur")
    R, C = cur.shape
    if prev is not None:
        _arr(prev, np.float32, (R, C), "prev")
    k_stride = k if k_stride is None else k_stride
    idx = np.full((R, k_stride), idx_fill, np.int32)
    counts = np.zeros(R, np.int32)
    _check(_load().oracle_topk_cols(_p(cur), _p(prev), R, C, C, k, _p(idx), _p(counts), k_stride),
           "oracle_topk_cols")
    return idx, counts


def mask_to_indices(mask, C, k_stride, idx_fill=-1):
    """mask [R, ld_words] uint32 (bit-packed rows) -> (idx [R, k_stride] int32, counts [R] int32).  App. B.4, Table 3."""
    _arr(mask, np.uint32, None, "mask")
    R, ld_words = mask.shape
    idx = np.full((R, k_stride), idx_fill, np.int32)
    counts = np.zeros(R, np.int32)
    _check(_load().oracle_mask_to_indices(_p(mask), ld_words, R, C, _p(idx), _p(counts), k_stride),
           "oracle_mask_to_indices")
    return idx, counts


def indices_to_mask(idx, counts, C, ld_words=None, fill=0):
    """idx [R, k_stride] int32, counts [R] int32 -> mask [R, ld_words] uint32 (bit-packed rows).  App. B.4."""
    _arr(idx, np.int32, None, "idx")
    R, k_stride = idx.shape
    _arr(counts, np.int32, (R,), "counts")
    ld_words = -(-C // 32) if ld_words is None else ld_words
    mask = np.full((R, ld_words), fill, np.uint32)
    _check(_load().oracle_indices_to_mask(_p(idx), _p(counts), R, C, k_stride, _p(mask), ld_words),
           "oracle_indices_to_mask")
    return mask


def attn_dense(q, k, v, c, scale, want_colsum=False):
    """q [B,H,Nq,E], k,v [B,H,Nk,E] float32 -> out float64 [B,H,Nq,E] (and D [B,H,NB,Nk])."""
    _arr(q, np.float32, None, "q")
    B, H, Nq, E = q.shape
    Nk = k.shape[2]
    _arr(k, np.float32, (B, H, Nk, E), "k")
    _arr(v, np.float32, (B, H, Nk, E), "v")
    NB = -(-Nq // c)
    out = np.empty((B, H, Nq, E), np.float64)
    D = np.empty((B, H, NB, Nk), np.float64) if want_colsum else None
    _check(_load().oracle_attn_dense(_p(q), _p(k), _p(v), _p(out), _p(D), B, H, Nq, Nk, E, c, float(scale)),
           "oracle_attn_dense")
    return (out, D) if want_colsum else out


def attn_row_stats(q, k, scale):
    """q [B,H,Nq,E], k [B,H,Nk,E] float32 -> (m, l) float64 [B,H,Nq]: row max of the scaled scores and
    sum_j exp(score - m).  The normalisers Alg. 4 carries between steps."""
    _arr(q, np.float32, None, "q")
    B, H, Nq, E = q.shape
    Nk = k.shape[2]
    _arr(k, np.float32, (B, H, Nk, E), "k")
    m = np.empty((B, H, Nq), np.float64)
    l = np.empty((B, H, Nq), np.float64)
    _check(_load().oracle_attn_row_stats(_p(q), _p(k), _p(m), _p(l), B, H, Nq, Nk, E, float(scale)),
           "oracle_attn_row_stats")
    return m, l


def attn_colsum_stale(q, k, prev_m, prev_l, c, scale):
    """cs[b,h,i,j] = sum over the rows n of chunk i of exp(scale q_n.k_j - prev_m[n]) / prev_l[n].  Alg. 4."""
    _arr(q, np.float32, None, "q")
    B, H, Nq, E = q.shape
    Nk = k.shape[2]
    _arr(k, np.float32, (B, H, Nk, E), "k")
    _arr(prev_m, np.float64, (B, H, Nq), "prev_m")
    _arr(prev_l, np.float64, (B, H, Nq), "prev_l")
    NB = -(-Nq // c)
    cs = np.empty((B, H, NB, Nk), np.float64)
    _check(_load().oracle_attn_colsum_stale(_p(q), _p(k), _p(prev_m), _p(prev_l), _p(cs), B, H, Nq, Nk, E, c,
                                            float(scale)), "oracle_attn_colsum_stale")
    return cs


def attn_sparse_delta(q, k, v, idx, counts, base, c, scale, o_scale):
    """out = base + o_scale * softmax_S(scale q k_S^T) v_S per query chunk.  Alg. 3."""
    _arr(q, np.float32, None, "q")
    B, H, Nq, E = q.shape
    Nk = k.shape[2]
    _arr(k, np.float32, (B, H, Nk, E), "k")
    _arr(v, np.float32, (B, H, Nk, E), "v")
    NB = -(-Nq // c)
    _arr(idx, np.int32, None, "idx")
    k_stride = idx.shape[-1]
    _arr(idx, np.int32, (B, H, NB, k_stride), "idx")
    _arr(counts, np.int32, (B, H, NB), "counts")
    _arr(base, np.float64, (B, H, Nq, E), "base")
    out = np.empty((B, H, Nq, E), np.float64)
    _check(_load().oracle_attn_sparse_delta(_p(q), _p(k), _p(v), _p(idx), _p(counts), _p(base), _p(out),
                                            B, H, Nq, Nk, E, c, k_stride, float(scale), float(o_scale)),
           "oracle_attn_sparse_delta")
    return out


def mlp_dense(x, w1, b1, w2, b2, c, act, a_ld=None, want_caches=True):
    """x [B,N,D], w1,w2 [F,D] -> out [B,N,D] float64 (+ a_cache [B,F,a_ld], T_m [B,NB,F]).  Alg. 5."""
    _arr(x, np.float32, None, "x")
    B, N, D = x.shape
    F = w1.shape[0]
    _arr(w1, np.float32, (F, D), "w1")
    _arr(w2, np.float32, (F, D), "w2")
    if b1 is not None:
        _arr(b1, np.float32, (F,), "b1")
    if b2 is not None:
        _arr(b2, np.float32, (D,), "b2")
    a_ld = N if a_ld is None else a_ld
    NB = -(-N // c)
    out = np.empty((B, N, D), np.float64)
    a_cache = np.zeros((B, F, a_ld), np.float64) if want_caches else None
    T_m = np.empty((B, NB, F), np.float64) if want_caches else None
    _check(_load().oracle_mlp_dense(_p(x), _p(w1), _p(b1), _p(w2), _p(b2), _p(out), _p(a_cache), a_ld,
                                    _p(T_m), B, N, D, F, c, act), "oracle_mlp_dense")
    return (out, a_cache, T_m) if want_caches else out


def mlp_tile_scores(x, w1, c):
    """T[b,i,:] = mean_c(x) @ w1^T, float64 [B,NB,F].  Alg. 7."""
    _arr(x, np.float32, None, "x")
    B, N, D = x.shape
    F = w1.shape[0]
    _arr(w1, np.float32, (F, D), "w1")
    NB = -(-N // c)
    T = np.empty((B, NB, F), np.float64)
    _check(_load().oracle_mlp_tile_scores(_p(x), _p(w1), _p(T), B, N, D, F, c), "oracle_mlp_tile_scores")
    return T


def mlp_sparse_delta(x, w1, b1, w2, idx, counts, a_cache, o_cache, c, act):
    """Updates a_cache [B,F,a_ld] and o_cache [B,N,D] (float64) in place.  Alg. 6."""
    _arr(x, np.float32, None, "x")
    B, N, D = x.shape
    F = w1.shape[0]
    _arr(w1, np.float32, (F, D), "w1")
    _arr(w2, np.float32, (F, D), "w2")
    if b1 is not None:
        _arr(b1, np.float32, (F,), "b1")
    NB = -(-N // c)
    _arr(idx, np.int32, None, "idx")
    k_stride = idx.shape[-1]
    _arr(idx, np.int32, (B, NB, k_stride), "idx")
    _arr(counts, np.int32, (B, NB), "counts")
    _arr(a_cache, np.float64, None, "a_cache")
    a_ld = a_cache.shape[2]
    _arr(a_cache, np.float64, (B, F, a_ld), "a_cache")
    _arr(o_cache, np.float64, (B, N, D), "o_cache")
    _check(_load().oracle_mlp_sparse_delta(_p(x), _p(w1), _p(b1), _p(w2), _p(idx), _p(counts), _p(a_cache),
                                           a_ld, _p(o_cache), B, N, D, F, c, k_stride, act),
           "oracle_mlp_sparse_delta")
    return a_cache, o_cache
