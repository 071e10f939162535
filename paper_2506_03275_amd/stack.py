"""A stack of DiT blocks over diffusion steps, sequenced through the C ABI (no arithmetic here).

Step 1 is dense and fills every cache (Alg. 2 and Alg. 5 of the paper): dense attention with exact column sums,
top-k of the column sums, O_cache = O_dense - delta (the sparse-delta call with o_scale = -1), dense MLP with A_cache
and M_cache, token-merged pre-activations T_m.  Later steps are column-sparse (Alg. 3, 6, 7): attention delta with the
cached indices, then T = mean_c(x) W1^T, top-k of |T - T_m|, MLP delta.  A later dense step (a cache refresh) takes
its column sums in the same kernel as the attention, against the softmax normalisers the previous dense step left
(Alg. 4), and leaves its own for the next refresh.

With `overlap`, the index computation of the NEXT block (scores GEMM + top-k, which depend only on that block's input
and weights) runs on a second stream beside the current block's attention and MLP delta; an event hands the indices
over.  In a real DiT the next block's input depends on this block's output, so that overlap is a property of a stack
with pre-generated inputs; what carries over to a model is that the index work needs no result of the delta kernels.
"""
import math

import torch

from . import (ACT_GELU_TANH, attn_dense, attn_dense_colsum_stale, attn_dense_row_stats,
               attn_dense_workspace_bytes, attn_sparse_delta, mlp_dense,
               mlp_sparse_delta, mlp_tile_mean_preact, mlp_tile_mean_workspace_bytes, mlp_workspace_bytes,
               topk_cols)


def _u8(nbytes, dev):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=dev)


class Block:
    """Caches, index lists and workspaces of one block (device tensors owned here)."""

    def __init__(self, inputs, c, k_attn, k_mlp, act=ACT_GELU_TANH):
        q, x, w1 = inputs["q"][0], inputs["x"][0], inputs["w1"]
        dev = q.device
        B, H, N, E = q.shape
        D, F = x.shape[-1], w1.shape[0]
        NB = -(-N // c)
        self.inputs, self.c, self.k_attn, self.k_mlp, self.act = inputs, c, k_attn, k_mlp, act
        self.B, self.H, self.N, self.E, self.D, self.F, self.NB = B, H, N, E, D, F, NB
        self.scale = 1.0 / math.sqrt(E)
        self.idx_a = torch.zeros((B, H, NB, max(k_attn, 1)), dtype=torch.int32, device=dev)
        self.cnt_a = torch.zeros((B, H, NB), dtype=torch.int32, device=dev)
        self.idx_m = torch.zeros((B, NB, max(k_mlp, 1)), dtype=torch.int32, device=dev)
        self.cnt_m = torch.zeros((B, NB), dtype=torch.int32, device=dev)
        self.o_cache = torch.empty_like(q)            # O_dense - delta of the dense step
        self.attn_out = torch.empty_like(q)
        self.a_cache = torch.zeros((B, F, -(-N // 8) * 8), dtype=torch.bfloat16, device=dev)
        self.m_cache = torch.empty_like(x)            # the MLP output, merged in place on sparse steps
        self.T_m = torch.empty((B, NB, F), dtype=torch.float32, device=dev)
        self.T = torch.empty_like(self.T_m)
        self.ws_tm = _u8(mlp_tile_mean_workspace_bytes(B, N, D, F, c), dev)
        self.ws_mlp = _u8(mlp_workspace_bytes(B, N, D, F, c, max(k_mlp, 1)), dev)
        self.row_m = torch.empty((B, H, N), dtype=torch.float32, device=dev)   # softmax normalisers of the last
        self.row_l = torch.empty_like(self.row_m)                              # dense step (valid once has_stats)
        self.has_stats = False

    def dense_step(self, step, colsum, ws_attn):
        """Alg. 2 + Alg. 5 on the inputs of `step`; colsum [B,H,NB,ld] fp32 and ws_attn are shared scratch."""
        i = self.inputs
        q, k, v, x = i["q"][step], i["k"][step], i["v"][step], i["x"][step]
        if self.has_stats:   # Alg. 4: one kernel; the normalisers are replaced row by row by the workgroup that read them
            attn_dense_colsum_stale(q, k, v, self.attn_out, self.row_m, self.row_l, colsum, self.c, self.scale,
                                    self.row_m, self.row_l)
        else:
            attn_dense(q, k, v, self.attn_out, colsum, self.c, self.scale, ws_attn)
            m, l = attn_dense_row_stats(ws_attn, self.B, self.H, self.N)
            self.row_m.copy_(m)
            self.row_l.copy_(l)
            self.has_stats = True
        topk_cols(colsum.view(-1, colsum.shape[-1])[:, :self.N], None, self.k_attn,
                  self.idx_a.view(-1, self.idx_a.shape[-1]), self.cnt_a.view(-1))
        attn_sparse_delta(q, k, v, self.idx_a, self.cnt_a, self.attn_out, self.o_cache, self.c, self.scale, -1.0)
        mlp_dense(x, i["w1"], i["b1"], i["w2"], i["b2"], self.m_cache, self.a_cache, self.c, self.act)
        mlp_tile_mean_preact(x, i["w1"], self.T_m, self.c, self.ws_tm)

    def mlp_indices(self, step):
        """Alg. 7: T = mean_c(x) W1^T, then top-k of |T - T_m|."""
        i = self.inputs
        mlp_tile_mean_preact(i["x"][step], i["w1"], self.T, self.c, self.ws_tm)
        topk_cols(self.T.view(-1, self.F), self.T_m.view(-1, self.F), self.k_mlp,
                  self.idx_m.view(-1, self.idx_m.shape[-1]), self.cnt_m.view(-1))

    def attn_delta(self, step):
        """Alg. 3 with the indices of the dense step."""
        i = self.inputs
        attn_sparse_delta(i["q"][step], i["k"][step], i["v"][step], self.idx_a, self.cnt_a, self.o_cache,
                          self.attn_out, self.c, self.scale, 1.0)

    def mlp_delta(self, step):
        """Alg. 6: GEMM1 on the selected neurons + cache update, GEMM2 + merge into M_cache."""
        i = self.inputs
        mlp_sparse_delta(i["x"][step], i["w1"], i["b1"], i["w2"], self.idx_m, self.cnt_m, self.a_cache, self.m_cache,
                         self.c, self.act, self.ws_mlp)


def dense_step(blocks, step=0):
    """Runs the dense step of every block on the current stream."""
    b0 = blocks[0]
    dev = b0.o_cache.device
    ld = -(-b0.N // 4) * 4
    colsum = torch.empty((b0.B, b0.H, b0.NB, ld), dtype=torch.float32, device=dev)
    ws_attn = _u8(attn_dense_workspace_bytes(b0.B, b0.H, b0.N), dev)
    for blk in blocks:
        blk.dense_step(step, colsum, ws_attn)


def sparse_step(blocks, step, side_stream=None, after_block=None):
    """Runs one column-sparse step of every block.  With side_stream, block b+1's MLP indices are computed on it
    while block b runs on the current stream.  after_block(b, blk), if given, is called after block b's calls were
    enqueued (tests use it to copy results out)."""
    main = torch.cuda.current_stream()
    if side_stream is None:
        for b, blk in enumerate(blocks):
            blk.attn_delta(step)
            blk.mlp_indices(step)
            blk.mlp_delta(step)
            if after_block:
                after_block(b, blk)
        return
    ready = [torch.cuda.Event() for _ in blocks]
    side_stream.wait_stream(main)        # everything enqueued so far (previous step's caches) is visible to the side stream
    with torch.cuda.stream(side_stream):
        blocks[0].mlp_indices(step)
        ready[0].record(side_stream)
    for b, blk in enumerate(blocks):
        if b + 1 < len(blocks):
            with torch.cuda.stream(side_stream):
                blocks[b + 1].mlp_indices(step)
                ready[b + 1].record(side_stream)
        blk.attn_delta(step)
        main.wait_event(ready[b])
        blk.mlp_delta(step)
        if after_block:
            after_block(b, blk)
    main.wait_stream(side_stream)
