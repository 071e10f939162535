"""Python binding of the gfx950 Chipmunk library (include/chipmunk.h).

Argument marshalling only: each function checks dtype, device and contiguity
of the torch tensors it is given, passes their device pointers and the current
HIP stream to the C entry point of the same name, and raises on a non-zero
status.  Every step of the method runs inside the HIP kernels; there is no CPU
or PyTorch fallback, and importing this package without the built library
fails loudly on first use.
"""
import ctypes
import os

import torch

from . import build as _build

_lib = None

_c_int = ctypes.c_int
_c_i64 = ctypes.c_int64
_c_f32 = ctypes.c_float
_c_ptr = ctypes.c_void_p
_c_size = ctypes.c_size_t

ACT_GELU_ERF = 0
ACT_GELU_TANH = 1

_SIGNATURES = {
    "chipmunk_voxel_reorder": ([_c_ptr] * 4 + [_c_int] * 11 + [_c_ptr], ctypes.c_int32),
    "chipmunk_topk_cols": ([_c_ptr, _c_ptr, _c_int, _c_int, _c_i64, _c_int, _c_ptr, _c_ptr, _c_int, _c_ptr],
                           ctypes.c_int32),
    "chipmunk_mask_to_indices": ([_c_ptr, _c_i64, _c_int, _c_int, _c_ptr, _c_ptr, _c_int, _c_ptr], ctypes.c_int32),
    "chipmunk_indices_to_mask": ([_c_ptr, _c_ptr, _c_int, _c_int, _c_int, _c_ptr, _c_i64, _c_ptr], ctypes.c_int32),
    "chipmunk_attn_sparse_delta": ([_c_ptr] * 7 + [_c_int] * 6 + [_c_f32, _c_f32, _c_ptr], ctypes.c_int32),
    "chipmunk_attn_block_sparse_delta": ([_c_ptr] * 7 + [_c_int] * 6 + [_c_f32, _c_f32, _c_ptr], ctypes.c_int32),
    "chipmunk_attn_dense_workspace_bytes": ([_c_int] * 3, _c_size),
    "chipmunk_attn_dense": ([_c_ptr] * 5 + [_c_i64] + [_c_int] * 5 + [_c_f32, _c_ptr, _c_size, _c_ptr],
                            ctypes.c_int32),
    "chipmunk_attn_colsum_stale": ([_c_ptr] * 5 + [_c_i64] + [_c_int] * 5 + [_c_f32, _c_ptr], ctypes.c_int32),
    "chipmunk_attn_dense_colsum_stale": ([_c_ptr] * 7 + [_c_i64] + [_c_ptr] * 2 + [_c_int] * 5 + [_c_f32, _c_ptr],
                                         ctypes.c_int32),
    "chipmunk_mlp_tile_mean_workspace_bytes": ([_c_int] * 5, _c_size),
    "chipmunk_mlp_tile_mean_preact": ([_c_ptr] * 3 + [_c_int] * 5 + [_c_ptr, _c_size, _c_ptr], ctypes.c_int32),
    "chipmunk_mlp_tile_mean_preact_static_capacity": ([], _c_size),
    "chipmunk_mlp_tile_mean_preact_static": ([_c_ptr] * 3 + [_c_int] * 5 + [_c_ptr], ctypes.c_int32),
    "chipmunk_mlp_workspace_bytes": ([_c_int] * 6, _c_size),
    "chipmunk_mlp_sparse_delta": ([_c_ptr] * 7 + [_c_i64, _c_ptr] + [_c_int] * 7 + [_c_ptr, _c_size, _c_ptr],
                                  ctypes.c_int32),
    "chipmunk_mlp_overlapped_workspace_bytes": ([_c_int] * 6, _c_size),
    "chipmunk_mlp_sparse_delta_overlapped": ([_c_ptr] * 7 + [_c_i64, _c_ptr] + [_c_int] * 7 + [_c_ptr, _c_size, _c_ptr],
                                             ctypes.c_int32),
    "chipmunk_mlp_dense": ([_c_ptr] * 7 + [_c_i64] + [_c_int] * 6 + [_c_ptr], ctypes.c_int32),
    "chipmunk_status_string": ([ctypes.c_int32], ctypes.c_char_p),
}

EXPORTED_SYMBOLS = tuple(_SIGNATURES)


def library_path():
    return _build.LIB


def load():
    """Load libchipmunk_hip.so (building it first only when it does not exist)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        lib = ctypes.CDLL(_build.LIB)
        for name, (argtypes, restype) in _SIGNATURES.items():
            fn = getattr(lib, name)  # AttributeError if the library lacks a declared symbol
            fn.argtypes = argtypes
            fn.restype = restype
        _lib = lib
    return _lib


class ChipmunkError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        text = load().chipmunk_status_string(self.status).decode()
        super().__init__(f"{where}: {text} (status {self.status})")


def _check(status, where):
    if status != 0:
        raise ChipmunkError(status, where)


def _ptr(t, dtype, name):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or t.dtype != dtype:
        raise TypeError(f"{name}: expected a torch tensor of {dtype}")
    if not t.is_cuda:
        raise ValueError(f"{name}: must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    return t.data_ptr()


def _ptr_rows(t, dtype, name):
    """A [R, C] tensor whose rows are dense but may be spaced by a leading dimension larger than C."""
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or t.dtype != dtype or t.dim() != 2:
        raise TypeError(f"{name}: expected a 2-D torch tensor of {dtype}")
    if not t.is_cuda:
        raise ValueError(f"{name}: must live on the GPU")
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError(f"{name}: rows must be dense")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def voxel_reorder(src, dst, perm, inv_perm, n_prefix, T, H, W, n_suffix, vt, vh, vw, inverse=False):
    """src, dst: [batch, N, ...] tensors of one dtype (or both None); perm, inv_perm: int32 [N] or None."""
    if (src is None) != (dst is None):
        raise ValueError("src and dst must both be given or both be None")
    batch, row_bytes, sp, dp = 0, 4, None, None
    if src is not None:
        if src.shape != dst.shape or src.dtype != dst.dtype:
            raise ValueError("src and dst must agree in shape and dtype")
        batch = src.shape[0]
        row_bytes = src.element_size() * int(src[0, 0].numel())
        sp, dp = _ptr(src, src.dtype, "src"), _ptr(dst, dst.dtype, "dst")
    _check(load().chipmunk_voxel_reorder(sp, dp, _ptr(perm, torch.int32, "perm"),
                                         _ptr(inv_perm, torch.int32, "inv_perm"), batch, n_prefix, T, H, W,
                                         n_suffix, vt, vh, vw, row_bytes, int(bool(inverse)), _stream()),
           "chipmunk_voxel_reorder")


def topk_cols(cur, prev, k, idx, counts):
    """cur, prev: fp32 [R, C] with dense rows and one common row stride (prev may be None); idx: int32
    [R, k_stride]; counts: int32 [R]."""
    R, C = cur.shape
    if prev is not None and (prev.shape != cur.shape or prev.stride(0) != cur.stride(0)):
        raise ValueError("prev must have the shape and row stride of cur")
    _check(load().chipmunk_topk_cols(_ptr_rows(cur, torch.float32, "cur"), _ptr_rows(prev, torch.float32, "prev"), R, C,
                                     cur.stride(0), k, _ptr(idx, torch.int32, "idx"),
                                     _ptr(counts, torch.int32, "counts"), idx.shape[-1], _stream()),
           "chipmunk_topk_cols")


def mask_to_indices(mask, C, idx, counts):
    """mask: int32 [R, ld_words] bit-packed rows; idx: int32 [R, k_stride]; counts: int32 [R] (both written)."""
    R, ld_words = mask.shape
    _check(load().chipmunk_mask_to_indices(_ptr(mask, torch.int32, "mask"), ld_words, R, C,
                                           _ptr(idx, torch.int32, "idx"), _ptr(counts, torch.int32, "counts"),
                                           idx.shape[-1], _stream()), "chipmunk_mask_to_indices")


def indices_to_mask(idx, counts, C, mask):
    """idx: int32 [R, k_stride]; counts: int32 [R]; mask: int32 [R, ld_words] bit-packed rows (written)."""
    R, ld_words = mask.shape
    _check(load().chipmunk_indices_to_mask(_ptr(idx, torch.int32, "idx"), _ptr(counts, torch.int32, "counts"), R, C,
                                           idx.shape[-1], _ptr(mask, torch.int32, "mask"), ld_words, _stream()),
           "chipmunk_indices_to_mask")


def attn_sparse_delta(q, k, v, idx, counts, base, out, c, softmax_scale, o_scale):
    """q,k,v,base,out: bf16 [B,H,N,E]; idx: int32 [B,H,NB,k_stride]; counts: int32 [B,H,NB]."""
    B, H, N, E = q.shape
    k_stride = 0 if idx is None else idx.shape[-1]
    bf = torch.bfloat16
    _check(load().chipmunk_attn_sparse_delta(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"),
                                             _ptr(idx, torch.int32, "idx"), _ptr(counts, torch.int32, "counts"),
                                             _ptr(base, bf, "base"), _ptr(out, bf, "out"), B, H, N, E, c,
                                             k_stride, float(softmax_scale), float(o_scale), _stream()),
           "chipmunk_attn_sparse_delta")


ATTN_BLOCK_COLUMNS = 128


def attn_block_sparse_delta(q, k, v, blocks, block_counts, base, out, c, softmax_scale, o_scale):
    """q,k,v,base,out: bf16 [B,H,N,E]; blocks: int32 [B,H,NB,kb_stride] (numbers of 128-column key blocks);
    block_counts: int32 [B,H,NB]."""
    B, H, N, E = q.shape
    bf = torch.bfloat16
    _check(load().chipmunk_attn_block_sparse_delta(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"),
                                                   _ptr(blocks, torch.int32, "blocks"),
                                                   _ptr(block_counts, torch.int32, "block_counts"),
                                                   _ptr(base, bf, "base"), _ptr(out, bf, "out"), B, H, N, E, c,
                                                   blocks.shape[-1], float(softmax_scale), float(o_scale), _stream()),
           "chipmunk_attn_block_sparse_delta")


def attn_dense_workspace_bytes(B, H, N):
    return int(load().chipmunk_attn_dense_workspace_bytes(B, H, N))


def attn_dense(q, k, v, out, colsum, c, softmax_scale, ws=None):
    """q,k,v,out: bf16 [B,H,N,E]; colsum: fp32 [B,H,NB,ld] or None; ws: uint8 workspace (needed with colsum)."""
    B, H, N, E = q.shape
    bf = torch.bfloat16
    ld = 0 if colsum is None else colsum.shape[-1]
    _check(load().chipmunk_attn_dense(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"), _ptr(out, bf, "out"),
                                      _ptr(colsum, torch.float32, "colsum"), ld, B, H, N, E, c,
                                      float(softmax_scale), _ptr(ws, torch.uint8, "ws"),
                                      0 if ws is None else ws.numel(), _stream()), "chipmunk_attn_dense")


def attn_dense_row_stats(ws, B, H, N):
    """Views of the row statistics (m, l), fp32 [B,H,N] each, that attn_dense with column sums left in ws."""
    stats = ws[: 2 * B * H * N * 4].view(torch.float32)
    return stats[: B * H * N].view(B, H, N), stats[B * H * N:].view(B, H, N)


def attn_colsum_stale(q, k, prev_m, prev_l, colsum, c, softmax_scale):
    """q,k: bf16 [B,H,N,E]; prev_m, prev_l: fp32 [B,H,N]; colsum: fp32 [B,H,NB,ld] (written)."""
    B, H, N, E = q.shape
    bf, f32 = torch.bfloat16, torch.float32
    _check(load().chipmunk_attn_colsum_stale(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(prev_m, f32, "prev_m"),
                                             _ptr(prev_l, f32, "prev_l"), _ptr(colsum, f32, "colsum"),
                                             colsum.shape[-1], B, H, N, E, c, float(softmax_scale), _stream()),
           "chipmunk_attn_colsum_stale")


def attn_dense_colsum_stale(q, k, v, out, prev_m, prev_l, colsum, c, softmax_scale, new_m=None, new_l=None):
    """Alg. 4 in one kernel.  q,k,v,out: bf16 [B,H,N,E]; prev_m, prev_l, new_m, new_l: fp32 [B,H,N]; colsum: fp32
    [B,H,NB,ld] (written)."""
    B, H, N, E = q.shape
    bf, f32 = torch.bfloat16, torch.float32
    _check(load().chipmunk_attn_dense_colsum_stale(_ptr(q, bf, "q"), _ptr(k, bf, "k"), _ptr(v, bf, "v"),
                                                   _ptr(out, bf, "out"), _ptr(prev_m, f32, "prev_m"),
                                                   _ptr(prev_l, f32, "prev_l"), _ptr(colsum, f32, "colsum"),
                                                   colsum.shape[-1], _ptr(new_m, f32, "new_m"),
                                                   _ptr(new_l, f32, "new_l"), B, H, N, E, c, float(softmax_scale),
                                                   _stream()), "chipmunk_attn_dense_colsum_stale")


def mlp_tile_mean_workspace_bytes(B, N, D, F, c):
    return int(load().chipmunk_mlp_tile_mean_workspace_bytes(B, N, D, F, c))


def mlp_tile_mean_preact(x, w1, T, c, ws):
    """x: bf16 [B,N,D]; w1: bf16 [F,D]; T: fp32 [B,NB,F]; ws: uint8 workspace."""
    B, N, D = x.shape
    F = w1.shape[0]
    bf = torch.bfloat16
    _check(load().chipmunk_mlp_tile_mean_preact(_ptr(x, bf, "x"), _ptr(w1, bf, "w1"), _ptr(T, torch.float32, "T"),
                                                B, N, D, F, c, _ptr(ws, torch.uint8, "ws"),
                                                0 if ws is None else ws.numel(), _stream()),
           "chipmunk_mlp_tile_mean_preact")


def mlp_tile_mean_preact_static(x, w1, T, c):
    """mlp_tile_mean_preact on the library's own fixed scratch array: no workspace argument, no allocation."""
    B, N, D = x.shape
    F = w1.shape[0]
    bf = torch.bfloat16
    _check(load().chipmunk_mlp_tile_mean_preact_static(_ptr(x, bf, "x"), _ptr(w1, bf, "w1"),
                                                       _ptr(T, torch.float32, "T"), B, N, D, F, c, _stream()),
           "chipmunk_mlp_tile_mean_preact_static")


def mlp_workspace_bytes(B, N, D, F, c, k_stride):
    return int(load().chipmunk_mlp_workspace_bytes(B, N, D, F, c, k_stride))


def mlp_sparse_delta(x, w1, b1, w2, idx, counts, a_cache, o_cache, c, act, ws):
    """x: bf16 [B,N,D]; w1,w2: bf16 [F,D]; a_cache: bf16 [B,F,a_ld]; o_cache: bf16 [B,N,D]; ws: uint8 workspace."""
    B, N, D = x.shape
    F = w1.shape[0]
    bf = torch.bfloat16
    _check(load().chipmunk_mlp_sparse_delta(_ptr(x, bf, "x"), _ptr(w1, bf, "w1"), _ptr(b1, bf, "b1"),
                                            _ptr(w2, bf, "w2"), _ptr(idx, torch.int32, "idx"),
                                            _ptr(counts, torch.int32, "counts"), _ptr(a_cache, bf, "a_cache"),
                                            a_cache.shape[-1], _ptr(o_cache, bf, "o_cache"), B, N, D, F, c,
                                            idx.shape[-1], int(act), _ptr(ws, torch.uint8, "ws"),
                                            0 if ws is None else ws.numel(), _stream()),
           "chipmunk_mlp_sparse_delta")


def mlp_overlapped_workspace_bytes(B, N, D, F, c, k_stride):
    return int(load().chipmunk_mlp_overlapped_workspace_bytes(B, N, D, F, c, k_stride))


def mlp_sparse_delta_overlapped(x, w1, b1, w2, idx, counts, a_cache, o_cache, c, act, ws):
    """mlp_sparse_delta with the cache write-back inside the second GEMM's launch (workspace twice as large)."""
    B, N, D = x.shape
    F = w1.shape[0]
    bf = torch.bfloat16
    _check(load().chipmunk_mlp_sparse_delta_overlapped(_ptr(x, bf, "x"), _ptr(w1, bf, "w1"), _ptr(b1, bf, "b1"),
                                                       _ptr(w2, bf, "w2"), _ptr(idx, torch.int32, "idx"),
                                                       _ptr(counts, torch.int32, "counts"), _ptr(a_cache, bf, "a_cache"),
                                                       a_cache.shape[-1], _ptr(o_cache, bf, "o_cache"), B, N, D, F, c,
                                                       idx.shape[-1], int(act), _ptr(ws, torch.uint8, "ws"),
                                                       0 if ws is None else ws.numel(), _stream()),
           "chipmunk_mlp_sparse_delta_overlapped")


def mlp_dense(x, w1, b1, w2, b2, out, a_cache, c, act):
    """x,out: bf16 [B,N,D]; w1,w2: bf16 [F,D]; b1 [F], b2 [D] bf16 or None; a_cache: bf16 [B,F,a_ld]."""
    B, N, D = x.shape
    F = w1.shape[0]
    bf = torch.bfloat16
    _check(load().chipmunk_mlp_dense(_ptr(x, bf, "x"), _ptr(w1, bf, "w1"), _ptr(b1, bf, "b1"), _ptr(w2, bf, "w2"),
                                     _ptr(b2, bf, "b2"), _ptr(out, bf, "out"), _ptr(a_cache, bf, "a_cache"),
                                     a_cache.shape[-1], B, N, D, F, c, int(act), _stream()),
           "chipmunk_mlp_dense")
