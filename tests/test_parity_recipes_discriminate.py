"""CPU-only proof that the GPU parity tests can fail on a wrong delta.

For every input recipe a GPU parity test of a merge (`out = base + update`) uses, the oracle alone forms the
reference and a mutant whose update is 10 % short, `base + 0.9 (ref - base)`, and the test's own metric must reject
the mutant: rel_err(mutant, ref, ref - base) > REL_TOL.  The recipes are the functions of tests/parity.py that the
GPU tests call, run here on the CPU generator (other draws, the same distributions and shapes); at the benchmark
shapes one head and a few chunks stand for the full launch, since every (batch, head, chunk) unit is independent
and its statistics do not depend on how many others there are.
"""
import math

import numpy as np
import pytest
import torch

import parity as recipes
import synth_inputs as si
from parity import REL_TOL, rel_err, short_update

CPU = "cpu"


def _rejects(base, ref):
    return rel_err(short_update(base, ref), ref, ref - base) > REL_TOL


def _attn_ref(oracle, q, kk, v, idx, counts, base, c, scale, o_scale):
    basen = si.np_f32(base).astype(np.float64)
    ref = oracle.attn_sparse_delta(si.np_f32(q), si.np_f32(kk), si.np_f32(v), idx.numpy(), counts.numpy(), basen, c,
                                   scale, o_scale)
    return basen, ref


def _attn_case(B, H, N, E, c, k, seed, ragged, order="ascending", base_mode="unit"):
    q, kk, v = recipes.attn_inputs(B, H, N, E, seed, CPU)
    NB = -(-N // c)
    idx, counts = recipes.attn_indices(B * H * NB, N, k, seed, CPU, ragged, order)
    base = recipes.attn_base((B, H, N, E), k, base_mode, seed, CPU)
    return q, kk, v, idx.view(B, H, NB, k).contiguous(), counts.view(B, H, NB).contiguous(), base


@pytest.mark.parametrize("B,H,N,E,c,k,ragged", [
    (1, 2, 1024, 64, 128, 256, False), (1, 2, 1000, 64, 128, 250, True), (1, 2, 1100, 128, 192, 100, True),
    (2, 3, 700, 128, 128, 333, True), (1, 1, 500, 64, 192, 77, True), (1, 1, 192, 128, 192, 192, False),
    (1, 1, 50, 128, 192, 7, False),
])
def test_small_attention_recipes_reject_a_short_delta(oracle, B, H, N, E, c, k, ragged):
    """Recipe of test_attn_sparse_delta_parity."""
    q, kk, v, idx, counts, base = _attn_case(B, H, N, E, c, k, 0, ragged)
    for o_scale in (1.0, -1.0):
        basen, ref = _attn_ref(oracle, q, kk, v, idx, counts, base, c, 1.0 / math.sqrt(E), o_scale)
        assert _rejects(basen, ref)


@pytest.mark.parametrize("order", ["shuffled", "duplicates"])
@pytest.mark.parametrize("B,H,N,E,c,k", [(1, 2, 700, 128, 192, 100), (1, 2, 1024, 64, 128, 77)])
def test_index_list_recipes_reject_a_short_delta(oracle, order, B, H, N, E, c, k):
    """Recipe of test_attn_index_list_is_taken_as_given; also: the duplicated columns change the answer by more
    than the tolerance, so a kernel that dropped the repeats would fail there."""
    q, kk, v, idx, counts, base = _attn_case(B, H, N, E, c, k, 21, True, order, "delta")
    scale = 1.0 / math.sqrt(E)
    basen, ref = _attn_ref(oracle, q, kk, v, idx, counts, base, c, scale, 1.0)
    assert _rejects(basen, ref)
    if order == "duplicates":
        dedup = idx.clone()
        dedup[..., k - k // 3:] = idx[..., :1]                      # repeats replaced by one more copy of column 0 ...
        cnt = torch.minimum(counts, torch.tensor(k - k // 3))       # ... and cut off: the list without its repeats
        _, ref_dedup = _attn_ref(oracle, q, kk, v, dedup, cnt.to(torch.int32), base, c, scale, 1.0)
        assert rel_err(ref_dedup, ref, ref - basen) > REL_TOL


@pytest.mark.parametrize("B,H,N,E,c,n_blocks,ragged", [
    (1, 2, 1024, 64, 128, 2, False), (1, 2, 1100, 128, 192, 3, True), (2, 2, 700, 128, 128, 2, True),
    (1, 1, 500, 64, 192, 4, True), (1, 1, 100, 128, 192, 1, False),
])
def test_block_list_recipes_reject_a_short_delta(oracle, B, H, N, E, c, n_blocks, ragged):
    """Recipe of test_attn_block_sparse_delta_parity; and the expansion of a block list is what its text says."""
    q, kk, v = recipes.attn_inputs(B, H, N, E, 4, CPU)
    NB = -(-N // c)
    blocks, bcounts = recipes.attn_block_lists(B * H * NB, N, n_blocks, 4, CPU, ragged)
    idxn, cntn = recipes.expand_block_lists(blocks.numpy(), bcounts.numpy(), N)
    for u in range(len(cntn)):                                        # every column of every listed block, cut at N
        want = np.concatenate([np.arange(b * 128, min(N, (b + 1) * 128)) for b in blocks[u, :bcounts[u]].tolist()] or
                              [np.zeros(0, np.int64)])
        assert cntn[u] == len(want) and np.array_equal(idxn[u, :cntn[u]], want)
    base = recipes.attn_base((B, H, N, E), max(int(cntn.max()), 1), "delta", 4, CPU)
    basen = si.np_f32(base).astype(np.float64)
    ref = oracle.attn_sparse_delta(si.np_f32(q), si.np_f32(kk), si.np_f32(v), idxn.reshape(B, H, NB, -1),
                                   cntn.reshape(B, H, NB), basen, c, 1.0 / math.sqrt(E), 1.0)
    assert _rejects(basen, ref)


def test_roundtrip_recipe_rejects_a_short_delta(oracle):
    """Recipe of test_attn_all_columns_equals_dense_and_cache_roundtrip (cache = dense - delta, then + delta)."""
    B, H, N, E, c = 1, 2, 520, 128, 192
    q, kk, v, idx, counts, _ = _attn_case(B, H, N, E, c, 60, 3, False)
    scale = 1.0 / math.sqrt(E)
    dense = si.np_bf16_round(oracle.attn_dense(si.np_f32(q), si.np_f32(kk), si.np_f32(v), c, scale))
    dense_t = torch.from_numpy(dense)
    dense_n, cache_ref = _attn_ref(oracle, q, kk, v, idx, counts, dense_t, c, scale, -1.0)
    assert _rejects(dense_n, cache_ref)
    cache_t = torch.from_numpy(si.np_bf16_round(cache_ref))
    cache_n, again_ref = _attn_ref(oracle, q, kk, v, idx, counts, cache_t, c, scale, 1.0)
    assert _rejects(cache_n, again_ref)


@pytest.mark.parametrize("name,sparse_k", [("flux", 323), ("hunyuan", 8082), ("wan", 5292)])
@pytest.mark.parametrize("mode", ["zero", "delta"])
def test_full_shape_attention_recipes_reject_a_short_delta(oracle, name, sparse_k, mode):
    """Recipe of _check_sampled_attn_units: one head and two chunks of the full-length sequence."""
    cfg = si.CONFIGS[name]
    E, c = cfg["E"], cfg["c"]
    N = si.config_tokens(cfg)
    q, kk, v = recipes.attn_inputs(1, 1, N, E, 0, CPU)
    idx, counts = recipes.attn_indices(2, N, sparse_k, 0, CPU)
    base = recipes.attn_base((1, 1, N, E), sparse_k, mode, 0, CPU)
    NB = -(-N // c)
    for u, i in enumerate((0, NB - 1)):
        rows = slice(i * c, min(N, (i + 1) * c))
        basen, ref = _attn_ref(oracle, q[:, :, rows].contiguous(), kk, v, idx[u].view(1, 1, 1, -1).contiguous(),
                               counts[u].view(1, 1, 1), base[:, :, rows].contiguous(), c, 1.0 / math.sqrt(E), 1.0)
        assert _rejects(basen, ref), (name, mode, i)
        # what the earlier recipe allowed, kept as a regression: on an N(0,1) cache a 15 % short delta passed
        if mode == "delta" and name != "flux":
            unit_base = si.np_f32(recipes.attn_base(tuple(basen.shape), sparse_k, "unit", 1, CPU)).astype(np.float64)
            hidden = unit_base + 0.85 * (ref - basen)
            assert rel_err(hidden, unit_base + (ref - basen)) <= REL_TOL


def _mlp_step(oracle, x2, w1, b1, w2, idx, counts, a_cache, o_cache, c, act):
    a_after, o_after = a_cache.copy(), o_cache.copy()
    oracle.mlp_sparse_delta(si.np_f32(x2), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), idx.numpy(), counts.numpy(),
                            a_after, o_after, c, act)
    return a_after, o_after


@pytest.mark.parametrize("B,N,D,F,c,k,act", [
    (1, 1024, 256, 1024, 128, 256, 1), (2, 500, 256, 320, 192, 100, 0), (1, 300, 128, 256, 128, 256, 1),
    (1, 192, 128, 128, 192, 1, 1),
])
def test_small_mlp_recipes_reject_a_short_delta(oracle, B, N, D, F, c, k, act):
    """Recipe of test_mlp_sparse_delta_parity (first of its two chained steps)."""
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 1, CPU)
    NB = -(-N // c)
    o_ref, a_ref, _ = oracle.mlp_dense(si.np_f32(x1), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), si.np_f32(b2), c, act,
                                       a_ld=-(-N // 8) * 8)
    o_cache = si.np_bf16_round(o_ref).astype(np.float64)
    a_cache = si.np_bf16_round(a_ref).astype(np.float64)
    idx, counts = recipes.mlp_indices(B * NB, F, k, 10, CPU, ragged=True)
    a_after, o_after = _mlp_step(oracle, x2, w1, b1, w2, idx.view(B, NB, k).contiguous(), counts.view(B, NB).contiguous(),
                                 a_cache, o_cache, c, act)
    assert _rejects(o_cache, o_after)
    # a GEMM2 that did nothing, and the cache with only 90 % of the activations' change, fail as well
    assert rel_err(o_cache, o_after, o_after - o_cache) > REL_TOL
    assert rel_err(short_update(a_cache, a_after)[..., :N], a_after[..., :N]) > REL_TOL


@pytest.mark.parametrize("name", ["flux", "hunyuan", "wan"])
def test_full_shape_mlp_recipes_reject_a_short_delta(oracle, name):
    """Recipe of test_mlp_full_shape_sampled_units: one chunk of tokens at the full widths D, F and kept count."""
    cfg = si.CONFIGS[name]
    D, F, c = cfg["D"], cfg["F"], cfg["c"]
    k = si.kept(F, cfg["mlp_keep"])
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(1, c, D, F, 2, CPU)
    o_ref, a_ref, _ = oracle.mlp_dense(si.np_f32(x1), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), si.np_f32(b2), c, 1)
    o_cache = si.np_bf16_round(o_ref).astype(np.float64)
    a_cache = si.np_bf16_round(a_ref).astype(np.float64)
    idx, counts = recipes.mlp_indices(1, F, k, 3, CPU)
    a_after, o_after = _mlp_step(oracle, x2, w1, b1, w2, idx.view(1, 1, k), counts.view(1, 1), a_cache, o_cache, c, 1)
    assert _rejects(o_cache, o_after)
    assert rel_err(o_cache, o_after, o_after - o_cache) > REL_TOL          # an untouched cache fails
    # regression on the old recipe (x2 = x1 + 0.01 N(0,1)): there an untouched cache passed the tolerance
    x_small = si.perturb_all(x1, si.generator(5, CPU))
    _, o_small = _mlp_step(oracle, x_small, w1, b1, w2, idx.view(1, 1, k), counts.view(1, 1), a_cache, o_cache, c, 1)
    assert rel_err(o_cache, o_small, o_small - o_cache) <= REL_TOL


def test_stack_and_smoke_recipes_reject_a_short_delta(oracle):
    """Recipes of tests/test_gpu_stack.py (Tiny blocks, x moving by N(0,1) per step) and of smoke() (Tiny, x2
    independent of x1): attention cache fill, attention delta and MLP delta of the first sparse step."""
    cfg = si.CONFIGS["tiny"]
    B, H, E, c, D, F = cfg["B"], cfg["H"], cfg["E"], cfg["c"], cfg["D"], cfg["F"]
    N = si.config_tokens(cfg)
    NB = -(-N // c)
    k_a, k_m = si.kept(N, cfg["attn_keep"]), si.kept(F, cfg["mlp_keep"])
    scale, act = 1.0 / math.sqrt(E), 1
    inp = si.stack_inputs(cfg, 1, 2, 5, CPU, x_sigma=1.0)[0]
    f32 = si.np_f32
    q, k, v = (f32(inp[n][0]) for n in "qkv")
    dense, colsum = oracle.attn_dense(q, k, v, c, scale, want_colsum=True)
    idx_a, cnt_a = oracle.topk_cols(colsum.reshape(-1, N).astype(np.float32), None, k_a)
    idx_a, cnt_a = idx_a.reshape(B, H, NB, k_a), cnt_a.reshape(B, H, NB)
    dense = si.np_bf16_round(dense).astype(np.float64)
    cache = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, dense, c, scale, -1.0)
    assert _rejects(dense, cache)
    cache = si.np_bf16_round(cache).astype(np.float64)
    q, k, v = (f32(inp[n][1]) for n in "qkv")
    out = oracle.attn_sparse_delta(q, k, v, idx_a, cnt_a, cache, c, scale, 1.0)
    assert _rejects(cache, out)
    w1, b1, w2, b2 = (f32(inp[n]) for n in ("w1", "b1", "w2", "b2"))
    for x1, x2 in ((inp["x"][0], inp["x"][1]), si.mlp_steps(B, N, D, 0, CPU, independent=True)):
        m_cache, a_cache, T_m = oracle.mlp_dense(f32(x1), w1, b1, w2, b2, c, act)
        T = oracle.mlp_tile_scores(f32(x2), w1, c)
        idx_m, cnt_m = oracle.topk_cols(T.reshape(-1, F).astype(np.float32), T_m.reshape(-1, F).astype(np.float32), k_m)
        m_after, a_after = m_cache.copy(), a_cache.copy()
        oracle.mlp_sparse_delta(f32(x2), w1, b1, w2, idx_m.reshape(B, NB, k_m), cnt_m.reshape(B, NB), a_after, m_after, c,
                                act)
        assert _rejects(m_cache, m_after)
        assert np.sqrt(np.mean((m_after - m_cache) ** 2)) >= 0.2 * np.sqrt(np.mean(m_after ** 2))
