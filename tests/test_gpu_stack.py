"""The layer stack (several DiT blocks over consecutive diffusion steps) at a small shape: two blocks over three diffusion steps (one dense, two
column-sparse), with and without the side-stream overlap of the MLP index work, against the oracle chained the
same way.  The blocks' MLP inputs move by N(0,1) per step (x_sigma = 1), so the MLP delta is of the size of the cached
output and a wrong delta cannot pass.  The oracle takes its index lists from the GPU run (top-k parity has its own bit-exact tests on a shared
score buffer; here a borderline column chosen differently from slightly different scores would change what is
compared), everything else it computes itself in fp64 from the same bf16 inputs."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from parity import REL_TOL, SCORE_TOL, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _run_gpu(cm, cfg, inputs, k_a, k_m, overlap):
    from paper_2506_03275_amd import stack
    blocks = [stack.Block(inp, cfg["c"], k_a, k_m) for inp in inputs]
    stack.dense_step(blocks, 0)
    torch.cuda.synchronize()
    for blk in blocks:
        blk.dense_out_copy = blk.attn_out.clone()     # the sparse steps reuse attn_out
    side = torch.cuda.Stream() if overlap else None
    record = {}
    for step in (1, 2):
        def grab(b, blk, step=step):
            # enqueue copies on the main stream: they see this block's results, not later ones
            record[(step, b)] = (blk.attn_out.clone(), blk.m_cache.clone(), blk.idx_m.clone(), blk.cnt_m.clone())
        stack.sparse_step(blocks, step, side, grab)
    torch.cuda.synchronize()
    return blocks, record


@pytest.mark.parametrize("overlap", [False, True])
def test_stack_matches_chained_oracle(oracle, overlap):
    import paper_2506_03275_amd as cm
    cm.load()
    cfg = si.CONFIGS["tiny"]
    c, E = cfg["c"], cfg["E"]
    N = si.config_tokens(cfg)
    k_a, k_m = si.kept(N, cfg["attn_keep"]), si.kept(cfg["F"], cfg["mlp_keep"])
    inputs = si.stack_inputs(cfg, 2, 3, 5, DEV, x_sigma=1.0)
    blocks, record = _run_gpu(cm, cfg, inputs, k_a, k_m, overlap)
    scale, act = 1.0 / math.sqrt(E), cm.ACT_GELU_TANH
    f32 = si.np_f32
    for b, (blk, inp) in enumerate(zip(blocks, inputs)):
        idx_a, cnt_a = blk.idx_a.cpu().numpy(), blk.cnt_a.cpu().numpy()
        # dense step
        q, k, v, x = (f32(inp[n][0]) for n in "qkvx")
        w1, b1, w2, b2 = (f32(inp[n]) for n in ("w1", "b1", "w2", "b2"))
        # every merge is compared with the oracle applied to the call's own bf16 base, under the one metric of
        # tests/parity.py (floor: the larger of the output's and the update's RMS)
        dense_gpu = f32(blk.dense_out_copy).astype(np.float64)
        assert rel_err(dense_gpu, oracle.attn_dense(q, k, v, c, scale)) <= REL_TOL, (overlap, b)
        o_cache = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, dense_gpu, c, scale, -1.0)
        cache_gpu = f32(blk.o_cache).astype(np.float64)
        assert rel_err(cache_gpu, o_cache, o_cache - dense_gpu) <= REL_TOL, (overlap, b)
        m_cache, a_cache, T_m = oracle.mlp_dense(x, w1, b1, w2, b2, c, act, a_ld=blk.a_cache.shape[-1])
        for step in (1, 2):
            g_attn, g_mlp, g_idx, g_cnt = record[(step, b)]
            q, k, v, x = (f32(inp[n][step]) for n in "qkvx")
            ref = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, cache_gpu, c, scale, 1.0)
            assert rel_err(f32(g_attn), ref, ref - cache_gpu) <= REL_TOL, (overlap, b, step)
            # the GPU's index choice must be the exact top-k of the GPU's own scores
            T_gpu = torch.empty_like(blk.T)
            cm.mlp_tile_mean_preact(inp["x"][step], inp["w1"], T_gpu, c, blk.ws_tm)
            ref_idx, ref_cnt = oracle.topk_cols(T_gpu.view(-1, cfg["F"]).cpu().numpy(),
                                                blk.T_m.view(-1, cfg["F"]).cpu().numpy(), k_m)
            assert np.array_equal(g_idx.view(-1, k_m).cpu().numpy(), ref_idx), (overlap, b, step)
            assert np.array_equal(g_cnt.view(-1).cpu().numpy(), ref_cnt)
            assert rel_err(T_gpu.cpu().numpy(), oracle.mlp_tile_scores(x, w1, c)) <= SCORE_TOL
            m_before = m_cache.copy()
            oracle.mlp_sparse_delta(x, w1, b1, w2, g_idx.cpu().numpy(), g_cnt.cpu().numpy(), a_cache, m_cache, c, act)
            assert rel_err(f32(g_mlp), m_cache, m_cache - m_before) <= REL_TOL, (overlap, b, step)
        assert rel_err(f32(blk.a_cache), a_cache) <= REL_TOL


def test_stack_overlap_equals_serial():
    """The two schedules enqueue the same kernels on the same data: results must agree bit for bit."""
    import paper_2506_03275_amd as cm
    cm.load()
    cfg = si.CONFIGS["tiny"]
    N = si.config_tokens(cfg)
    k_a, k_m = si.kept(N, cfg["attn_keep"]), si.kept(cfg["F"], cfg["mlp_keep"])
    inputs = si.stack_inputs(cfg, 3, 3, 9, DEV, x_sigma=1.0)
    _, serial = _run_gpu(cm, cfg, inputs, k_a, k_m, False)
    _, overlapped = _run_gpu(cm, cfg, inputs, k_a, k_m, True)
    for key in serial:
        for a, b in zip(serial[key], overlapped[key]):
            assert torch.equal(a, b), key


def test_stack_sparse_step_as_hip_graph():
    """The sparse step is kernel launches only (no allocation, no memset, no host wait), so it can be captured as one
    HIP graph.  Every replay, with eager steps and synchronisations in between, must reproduce the eager result."""
    import paper_2506_03275_amd as cm
    from paper_2506_03275_amd import stack
    cm.load()
    cfg = si.CONFIGS["tiny"]
    N = si.config_tokens(cfg)
    k_a, k_m = si.kept(N, cfg["attn_keep"]), si.kept(cfg["F"], cfg["mlp_keep"])
    inputs = si.stack_inputs(cfg, 2, 3, 11, DEV, x_sigma=1.0)
    blocks = [stack.Block(inp, cfg["c"], k_a, k_m) for inp in inputs]
    stack.dense_step(blocks, 0)
    torch.cuda.synchronize()
    saved = [(blk.a_cache.clone(), blk.m_cache.clone()) for blk in blocks]

    def restore():                      # the step merges into the MLP caches in place
        for blk, (a, m) in zip(blocks, saved):
            blk.a_cache.copy_(a)
            blk.m_cache.copy_(m)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for blk in blocks for t in (blk.attn_out, blk.m_cache, blk.a_cache, blk.idx_m, blk.cnt_m)]

    def same(a, b):
        return all(torch.equal(x, y) for x, y in zip(a, b))

    stack.sparse_step(blocks, 1)
    eager = snapshot()
    restore()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stack.sparse_step(blocks, 1)
    for replay in range(3):
        restore()
        torch.cuda.synchronize()
        graph.replay()
        assert same(snapshot(), eager), f"replay {replay}"
        restore()
        stack.sparse_step(blocks, 1)    # eager work between the replays
        assert same(snapshot(), eager), f"eager run after replay {replay}"


def test_stack_dense_refresh_with_stale_normalisers(oracle):
    """Dense step, sparse step, a second dense step (the cache refresh, Alg. 4: column sums against the first
    dense step's normalisers, in the attention kernel), sparse step with the refreshed indices."""
    import paper_2506_03275_amd as cm
    from paper_2506_03275_amd import stack
    cm.load()
    cfg = si.CONFIGS["tiny"]
    c, E = cfg["c"], cfg["E"]
    N = si.config_tokens(cfg)
    k_a, k_m = si.kept(N, cfg["attn_keep"]), si.kept(cfg["F"], cfg["mlp_keep"])
    inputs = si.stack_inputs(cfg, 2, 4, 13, DEV, x_sigma=1.0)
    blocks = [stack.Block(inp, c, k_a, k_m) for inp in inputs]
    scale = 1.0 / math.sqrt(E)
    f32 = si.np_f32
    stack.dense_step(blocks, 0)
    stack.sparse_step(blocks, 1)
    torch.cuda.synchronize()
    ld = -(-N // 4) * 4
    ws = torch.empty(max(cm.attn_dense_workspace_bytes(cfg["B"], cfg["H"], N), 16), dtype=torch.uint8, device=DEV)
    for b, (blk, inp) in enumerate(zip(blocks, inputs)):
        assert blk.has_stats
        m0, l0 = blk.row_m.cpu().numpy().astype(np.float64), blk.row_l.cpu().numpy().astype(np.float64)
        idx_before = blk.idx_a.clone()
        colsum = torch.empty((cfg["B"], cfg["H"], blk.NB, ld), dtype=torch.float32, device=DEV)
        blk.dense_step(2, colsum, ws)
        torch.cuda.synchronize()
        q, k, v = (f32(inp[n][2]) for n in "qkv")
        dense_gpu = f32(blk.attn_out).astype(np.float64)
        assert rel_err(dense_gpu, oracle.attn_dense(q, k, v, c, scale)) <= REL_TOL, b
        got = colsum.cpu().numpy()[..., :N]
        assert rel_err(got.astype(np.float64), oracle.attn_colsum_stale(q, k, m0, l0, c, scale)) <= REL_TOL, b
        # the refreshed index lists are the exact top-k of the GPU's own column sums
        ref_idx, ref_cnt = oracle.topk_cols(got.reshape(-1, N), None, k_a)
        idx_a, cnt_a = blk.idx_a.cpu().numpy(), blk.cnt_a.cpu().numpy()
        assert np.array_equal(idx_a.reshape(-1, k_a), ref_idx) and np.array_equal(cnt_a.reshape(-1), ref_cnt)
        assert not torch.equal(idx_before, blk.idx_a)       # the inputs moved: so did the choice
        # the statistics left for the next refresh are this step's own
        m_ref, l_ref = oracle.attn_row_stats(q, k, scale)
        lse = blk.row_m.cpu().numpy().astype(np.float64) + np.log(blk.row_l.cpu().numpy().astype(np.float64))
        assert np.abs(lse - (m_ref + np.log(l_ref))).max() <= 2e-3
        cache_gpu = f32(blk.o_cache).astype(np.float64)
        o_cache = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, dense_gpu, c, scale, -1.0)
        assert rel_err(cache_gpu, o_cache, o_cache - dense_gpu) <= REL_TOL, b
        blk.attn_delta(3)
        torch.cuda.synchronize()
        q, k, v = (f32(inp[n][3]) for n in "qkv")
        ref = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, cache_gpu, c, scale, 1.0)
        assert rel_err(f32(blk.attn_out), ref, ref - cache_gpu) <= REL_TOL, b
