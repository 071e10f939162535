"""GPU-vs-oracle parity on seeded random small problems, through the C ABI.

The committed shapes of tests/test_gpu_parity.py are chosen by hand; here shapes, counts and options are drawn from a
seeded generator, one problem per test case, so that combinations nobody thought of get compared as well: a count
per unit anywhere in [0, k], every list order, both signs of o_scale, the three bases, padded cache rows, both forms
of the activation-cache write-back.  Same metric and tolerance as everywhere (tests/parity.py); every attention case
is also run twice on the same inputs and must agree bit for bit.  The top-k, the mask conversions and the reorder are
compared bit for bit with the oracle on random row lengths (both sides of the short-row limit), score distributions
with and without ties, padded rows, and grids whose voxels divide nothing or are larger than the grid.
"""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
import parity as recipes
from parity import REL_TOL, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda"
SEED = 6
CASES = 24


@pytest.fixture(scope="module")
def cm():
    import paper_2506_03275_amd as cm
    cm.load()
    return cm


def _rng(case, stream):
    return np.random.default_rng([SEED, case, stream])


@pytest.mark.parametrize("case", range(CASES))
def test_attention_random_problem(cm, oracle, case):
    rng = _rng(case, 0)
    E = int(rng.choice([64, 128]))
    c = int(rng.choice([128, 192]))
    B, H = int(rng.integers(1, 3)), int(rng.integers(1, 4))
    N = int(rng.integers(1, 900))
    NB = -(-N // c)
    k = int(rng.integers(1, min(N, 400) + 1))
    seed = int(rng.integers(0, 1 << 20))
    mode = str(rng.choice(["zero", "delta", "unit"]))
    order = str(rng.choice(["ascending", "shuffled", "duplicates"]))
    o_scale = float(rng.choice([1.0, -1.0]))
    scale = 1.0 / math.sqrt(E)
    q, kk, v = recipes.attn_inputs(B, H, N, E, seed, DEV)
    base = recipes.attn_base(tuple(q.shape), k, mode, seed, DEV)
    idx, _ = recipes.attn_indices(B * H * NB, N, k, seed, DEV, order=order)
    idx = idx.view(B, H, NB, k).contiguous()
    counts = torch.from_numpy(rng.integers(0, k + 1, size=(B, H, NB)).astype(np.int32)).to(DEV)
    out = torch.empty_like(q)
    cm.attn_sparse_delta(q, kk, v, idx, counts, base, out, c, scale, o_scale)
    again = torch.full_like(q, 7.0)
    cm.attn_sparse_delta(q, kk, v, idx, counts, base, again, c, scale, o_scale)
    assert torch.equal(out, again)
    qn, kn, vn = si.np_f32(q), si.np_f32(kk), si.np_f32(v)
    basen = si.np_f32(base).astype(np.float64)
    ref = oracle.attn_sparse_delta(qn, kn, vn, idx.cpu().numpy(), counts.cpu().numpy(), basen, c, scale, o_scale)
    assert rel_err(si.np_f32(out), ref, ref - basen) <= REL_TOL
    # the same inputs through the every-column mode
    dense = torch.empty_like(q)
    cm.attn_sparse_delta(q, kk, v, None, None, None, dense, c, scale, 1.0)
    assert rel_err(si.np_f32(dense), oracle.attn_dense(qn, kn, vn, c, scale)) <= REL_TOL


@pytest.mark.parametrize("case", range(CASES))
def test_mlp_random_problem(cm, oracle, case):
    rng = _rng(case, 1)
    c = int(rng.choice([128, 192]))
    B = int(rng.integers(1, 3))
    N = int(rng.integers(1, 700))
    NB = -(-N // c)
    D = 128 * int(rng.integers(1, 4))
    F = 64 * int(rng.integers(1, 9))
    k = int(rng.integers(1, F + 1))
    act = int(rng.integers(0, 2))
    seed = int(rng.integers(0, 1 << 20))
    a_ld = -(-N // 8) * 8 + 8 * int(rng.integers(0, 3))              # cache rows may be longer than the sequence
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, seed, DEV)
    x1n, x2n, w1n, b1n, w2n, b2n = (si.np_f32(t) for t in (x1, x2, w1, b1, w2, b2))
    o_ref, a_ref, _ = oracle.mlp_dense(x1n, w1n, b1n, w2n, b2n, c, act, a_ld=a_ld)
    out = torch.empty_like(x1)
    a_dense = torch.zeros((B, F, a_ld), dtype=torch.bfloat16, device=DEV)
    cm.mlp_dense(x1, w1, b1, w2, b2, out, a_dense, c, act)
    assert rel_err(si.np_f32(out), o_ref) <= REL_TOL
    assert rel_err(si.np_f32(a_dense)[..., :N], a_ref[..., :N]) <= REL_TOL
    # one sparse step on caches that hold the oracle's dense step in the bf16 storage format
    o_cache = torch.from_numpy(o_ref).to(torch.bfloat16).to(DEV)
    a_cache = torch.from_numpy(a_ref).to(torch.bfloat16).to(DEV)
    o_ref = si.np_f32(o_cache).astype(np.float64)
    a_ref = si.np_f32(a_cache).astype(np.float64)
    idx, _ = recipes.mlp_indices(B * NB, F, k, seed + 1, DEV)
    idx = idx.view(B, NB, k).contiguous()
    counts = torch.from_numpy(rng.integers(0, k + 1, size=(B, NB)).astype(np.int32)).to(DEV)
    deferred = bool(rng.integers(0, 2))
    ws_bytes = (cm.mlp_overlapped_workspace_bytes if deferred else cm.mlp_workspace_bytes)(B, N, D, F, c, k)
    ws = torch.empty(max(int(ws_bytes), 16), dtype=torch.uint8, device=DEV)
    a_before, o_before = a_cache.clone(), o_ref.copy()
    step = cm.mlp_sparse_delta_overlapped if deferred else cm.mlp_sparse_delta
    step(x2, w1, b1, w2, idx, counts, a_cache, o_cache, c, act, ws)
    oracle.mlp_sparse_delta(x2n, w1n, b1n, w2n, idx.cpu().numpy(), counts.cpu().numpy(), a_ref, o_ref, c, act)
    assert rel_err(si.np_f32(a_cache)[..., :N], a_ref[..., :N]) <= REL_TOL
    assert rel_err(si.np_f32(o_cache), o_ref, o_ref - o_before) <= REL_TOL
    touched = torch.zeros((B, F, a_ld), dtype=torch.bool, device=DEV)
    for b in range(B):
        for i in range(NB):
            sel = idx[b, i, :int(counts[b, i])].long()
            touched[b, sel, i * c:min(N, (i + 1) * c)] = True
    assert torch.equal(a_cache[~touched], a_before[~touched])        # unselected cells, bit for bit


# The index and byte work: bit-exact against the oracle, so nothing here depends on a tolerance.

def _scores(rng, kind, R, C):
    if kind == "normal":
        return rng.standard_normal((R, C)).astype(np.float32)
    if kind == "quantised":                                          # a few dozen distinct values: ties decide
        return (np.round(rng.standard_normal((R, C)) * 4) / 4).astype(np.float32)
    if kind == "heavy_tail":
        return np.exp(3 * rng.standard_normal((R, C))).astype(np.float32)
    if kind == "narrow":                                             # a range of a few hundred ulps
        return (1.0 + 3e-5 * rng.random((R, C))).astype(np.float32)
    a = np.zeros((R, C), np.float32)                                 # "spikes": almost everything ties at zero
    a[:, rng.integers(0, C, size=max(1, C // 50))] = rng.random(max(1, C // 50)).astype(np.float32)
    return a


@pytest.mark.parametrize("case", range(CASES))
def test_topk_random_problem(cm, oracle, case):
    rng = _rng(case, 2)
    C = int(np.exp(rng.uniform(0.0, np.log(140000.0))))              # short rows (kept in LDS) and long ones
    R = int(rng.integers(1, 5))
    k = max(1, int(C * rng.choice([0.003, 0.07, 0.25, 0.5, 0.93, 1.0])))
    kind = str(rng.choice(["normal", "quantised", "heavy_tail", "narrow", "spikes"]))
    with_prev = bool(rng.integers(0, 2))
    ld = -(-C // 4) * 4 + 4 * int(rng.integers(0, 3))
    pad = int(rng.integers(0, 4))                                    # the list's row may be longer than k

    def rows(a):
        full = torch.zeros((R, ld), dtype=torch.float32, device=DEV)
        full[:, :C] = torch.from_numpy(a).to(DEV)
        return full

    cur_n = _scores(rng, kind, R, C)
    prev_n = _scores(rng, "quantised" if kind == "quantised" else "normal", R, C) if with_prev else None
    cur, prev = rows(cur_n), (rows(prev_n) if with_prev else None)
    idx = torch.full((R, k + pad), -7, dtype=torch.int32, device=DEV)
    counts = torch.full((R,), -7, dtype=torch.int32, device=DEV)
    cm.load().chipmunk_topk_cols(cur.data_ptr(), None if prev is None else prev.data_ptr(), R, C, ld, k,
                                 idx.data_ptr(), counts.data_ptr(), k + pad, None)
    torch.cuda.synchronize()
    ref_idx, ref_counts = oracle.topk_cols(cur_n, prev_n, k, k_stride=k + pad, idx_fill=-7)
    assert np.array_equal(counts.cpu().numpy(), ref_counts)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


@pytest.mark.parametrize("case", range(CASES))
def test_masks_random_problem(cm, oracle, case):
    rng = _rng(case, 3)
    C = int(np.exp(rng.uniform(0.0, np.log(200000.0))))
    R = int(rng.integers(1, 7))
    k = int(rng.integers(1, C + 1)) if C < 3000 else int(rng.integers(1, 3000))
    pad = int(rng.integers(0, 3))
    idx, _ = si.uniform_indices(R, C, k, int(rng.integers(0, 1 << 20)), DEV, k_stride=k + pad)
    counts = torch.from_numpy(rng.integers(0, k + 1, size=(R,)).astype(np.int32)).to(DEV)
    words = -(-C // 32)
    ld = words + int(rng.integers(0, 3))
    mask = torch.full((R, ld), -1, dtype=torch.int32, device=DEV)
    cm.indices_to_mask(idx, counts, C, mask)
    ref_mask = oracle.indices_to_mask(idx.cpu().numpy(), counts.cpu().numpy(), C, ld_words=ld, fill=0xffffffff)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), ref_mask)
    room = max(1, int(rng.integers(k // 2, k + 3)))                  # sometimes shorter than a row's population
    back = torch.full((R, room), -7, dtype=torch.int32, device=DEV)
    back_counts = torch.full((R,), -7, dtype=torch.int32, device=DEV)
    cm.mask_to_indices(mask, C, back, back_counts)
    ref_idx, ref_counts = oracle.mask_to_indices(ref_mask, C, room, idx_fill=-7)
    assert np.array_equal(back_counts.cpu().numpy(), ref_counts)
    assert np.array_equal(back.cpu().numpy(), ref_idx)


@pytest.mark.parametrize("case", range(CASES))
def test_voxel_reorder_random_geometry(cm, oracle, case):
    rng = _rng(case, 4)
    T, H, W = (int(x) for x in rng.integers(1, 14, size=3))
    vt, vh, vw = (int(x) for x in rng.integers(1, 6, size=3))
    npre, nsuf = int(rng.integers(0, 20)), int(rng.integers(0, 20))
    geom = (npre, T, H, W, nsuf, vt, vh, vw)
    N = npre + T * H * W + nsuf
    perm_ref, inv_ref = oracle.voxel_perm(*geom)
    perm = torch.full((N,), -1, dtype=torch.int32, device=DEV)
    inv = torch.full((N,), -1, dtype=torch.int32, device=DEV)
    cm.voxel_reorder(None, None, perm, inv, *geom)
    assert np.array_equal(perm.cpu().numpy(), perm_ref)
    assert np.array_equal(inv.cpu().numpy(), inv_ref)
    width = int(rng.choice([8, 24, 3, 1]))                           # 16-byte rows and rows of a few dwords
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (2, N, width), device=DEV, dtype=torch.int64,
                        generator=si.generator(case, DEV)).to(torch.int32)
    dst = torch.empty_like(src)
    cm.voxel_reorder(src, dst, None, None, *geom, inverse=False)
    raw = src.view(torch.uint8).cpu().numpy().reshape(2, N, -1)
    assert np.array_equal(dst.view(torch.uint8).cpu().numpy().reshape(2, N, -1),
                          oracle.reorder_rows(raw, perm_ref, inverse=False))
    back = torch.empty_like(src)
    cm.voxel_reorder(dst, back, None, None, *geom, inverse=True)
    assert torch.equal(back, src)
