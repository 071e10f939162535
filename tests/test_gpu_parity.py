"""GPU-vs-oracle parity, through the C ABI (via the thin Python binding).

Bit-exact for permutations and selected indices; max relative error <= 2e-2
(metric in tests/parity.py) for bf16 outputs computed with fp32 accumulation.
Small cases are compared element by element over the whole tensor; at the full
benchmark shapes the GPU runs the launch configuration bench.py times and
sampled units (a unit = one (batch, head, chunk) or (batch, chunk), which the
method treats independently) are compared one by one.
"""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
import parity as recipes
from parity import REL_TOL, SCORE_TOL, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda"


@pytest.fixture(scope="module")
def cm():
    import paper_2506_03275_amd as cm
    cm.load()
    return cm


def _u8(nbytes):
    return torch.empty(max(int(nbytes), 16), dtype=torch.uint8, device=DEV)


# ------------------------------------------------------------------ reorder ---

@pytest.mark.parametrize("geom", [
    (0, 8, 8, 16, 0, 4, 4, 8),        # Tiny
    (512, 1, 64, 64, 0, 1, 8, 8),     # FLUX-shaped
    (0, 30, 48, 80, 256, 4, 6, 8),    # HunyuanVideo-shaped (T does not divide)
    (0, 21, 45, 80, 0, 4, 6, 8),      # WAN-shaped (T, H do not divide)
    (3, 5, 7, 9, 2, 2, 3, 4),         # nothing divides
    (0, 1, 1, 1, 0, 1, 1, 1),         # one token
])
def test_voxel_reorder_bit_exact(cm, oracle, geom):
    npre, T, H, W, nsuf, vt, vh, vw = geom
    N = npre + T * H * W + nsuf
    perm_ref, inv_ref = oracle.voxel_perm(*geom)
    perm = torch.full((N,), -1, dtype=torch.int32, device=DEV)
    inv = torch.full((N,), -1, dtype=torch.int32, device=DEV)
    cm.voxel_reorder(None, None, perm, inv, npre, T, H, W, nsuf, vt, vh, vw)
    assert np.array_equal(perm.cpu().numpy(), perm_ref)
    assert np.array_equal(inv.cpu().numpy(), inv_ref)
    # data: 16-byte rows path (bf16 x 24) and 4-byte path (int32 x 3), batch 2
    g = si.generator(1, DEV)
    for shape, dtype in (((2, N, 24), torch.bfloat16), ((2, N, 3), torch.int32)):
        if dtype == torch.int32:
            src = torch.randint(-2 ** 31, 2 ** 31 - 1, shape, generator=g, device=DEV, dtype=torch.int64).to(torch.int32)
        else:
            src = si.randn_bf16(shape, g)
        dst = torch.empty_like(src)
        cm.voxel_reorder(src, dst, None, None, npre, T, H, W, nsuf, vt, vh, vw, inverse=False)
        raw = src.view(torch.uint8).cpu().numpy() if dtype == torch.int32 else src.view(torch.int16).cpu().numpy()
        got = dst.view(torch.uint8).cpu().numpy() if dtype == torch.int32 else dst.view(torch.int16).cpu().numpy()
        ref = oracle.reorder_rows(raw.reshape(2, N, -1), perm_ref, inverse=False)
        assert np.array_equal(got.reshape(2, N, -1), ref)
        back = torch.empty_like(src)
        cm.voxel_reorder(dst, back, None, None, npre, T, H, W, nsuf, vt, vh, vw, inverse=True)
        assert torch.equal(back, src)


# -------------------------------------------------------------------- top-k ---

@pytest.mark.parametrize("R,C,k,with_prev", [
    (16, 1024, 256, False),      # Tiny attention
    (8, 1024, 256, True),        # Tiny MLP
    (5, 1000, 1000, False),      # k = C
    (5, 1001, 1, True),          # k = 1, C % 4 != 0 (ld padded)
    (3, 7, 3, False),
    (24, 12288, 1229, True),     # FLUX MLP (row kept in LDS)
    (6, 13824, 968, True),       # WAN MLP
    (4, 14209, 100, False),      # just past the LDS limit: streaming path
    (12, 4608, 323, False),      # FLUX attention
    (3, 115456, 8082, False),    # HunyuanVideo attention row length
    (3, 75600, 5292, True),
    (2, 30000, 30000, False),    # long row, k = C
    (2, 30001, 1, False),        # long row, k = 1, C % 4 != 0
    (2, 50000, 25000, True),     # long row, half kept: the widest candidate bracket
    (2, 40000, 39990, False),
    (1, 800000, 5000, False),    # the column mask takes most of LDS
    (1, 1300000, 5000, True),    # beyond the single-pass limit: histogram passes over global memory
])
def test_topk_bit_exact(cm, oracle, R, C, k, with_prev):
    g = si.generator(7, DEV)
    ld = -(-C // 4) * 4
    cur = torch.zeros((R, ld), dtype=torch.float32, device=DEV)
    cur[:, :C] = torch.randn((R, C), generator=g, device=DEV)
    prev = None
    if with_prev:
        prev = torch.zeros((R, ld), dtype=torch.float32, device=DEV)
        prev[:, :C] = cur[:, :C] + 0.1 * torch.randn((R, C), generator=g, device=DEV)
    idx = torch.full((R, k + 3), -7, dtype=torch.int32, device=DEV)
    counts = torch.full((R,), -7, dtype=torch.int32, device=DEV)
    cm.load().chipmunk_topk_cols(cur.data_ptr(), None if prev is None else prev.data_ptr(), R, C, ld, k,
                                 idx.data_ptr(), counts.data_ptr(), k + 3, None)
    torch.cuda.synchronize()
    ref_idx, ref_counts = oracle.topk_cols(np.ascontiguousarray(cur[:, :C].cpu().numpy()),
                                           None if prev is None else np.ascontiguousarray(prev[:, :C].cpu().numpy()),
                                           k, k_stride=k + 3, idx_fill=-7)
    assert np.array_equal(counts.cpu().numpy(), ref_counts)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


def test_topk_ties_and_structured_scores(cm, oracle):
    """Heavy ties (quantised scores, zeros of both signs, constant rows) and the column-sum-like
    distribution of the attention case: the tie rule (lower column wins) decides many picks."""
    g = si.generator(11, DEV)
    R, C = 6, 20000
    cur = torch.round(torch.randn((R, C), generator=g, device=DEV) * 4) / 4      # ~30 distinct values
    cur[1] = 0.0
    cur[2, ::3] = -0.0
    cur[3] = torch.softmax(torch.randn((C,), generator=g, device=DEV) * 3, dim=0) * 192
    for k in (1, 17, 1400, C - 1):
        idx = torch.zeros((R, k), dtype=torch.int32, device=DEV)
        counts = torch.zeros((R,), dtype=torch.int32, device=DEV)
        cm.topk_cols(cur, None, k, idx, counts)
        ref_idx, _ = oracle.topk_cols(cur.cpu().numpy(), None, k)
        assert np.array_equal(idx.cpu().numpy(), ref_idx)
    prev = torch.round(torch.randn((R, C), generator=g, device=DEV) * 4) / 4
    idx = torch.zeros((R, 500), dtype=torch.int32, device=DEV)
    counts = torch.zeros((R,), dtype=torch.int32, device=DEV)
    cm.topk_cols(cur, prev, 500, idx, counts)
    ref_idx, _ = oracle.topk_cols(cur.cpu().numpy(), prev.cpu().numpy(), 500)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)


@pytest.mark.parametrize("kind", ["constant", "two_values", "tiny_range", "denormal", "negative", "infinities",
                                  "ascending", "descending", "spikes", "signed_zeros", "heavy_tail"])
def test_topk_long_rows_awkward_distributions(cm, oracle, kind):
    """Long rows whose scores give the single-pass selection nothing to hold on to: one value (every sample key
    equal, the whole row between the pivots), two values, a range of a few ulps, denormals, negative scores,
    infinities among the sample, sorted rows, a few spikes over zeros, zeros of both signs, a heavy tail.  With and
    without a previous score tensor, keep fractions from one column to all but one."""
    rng = np.random.default_rng(7)
    R, C = 3, 70001                                     # not a multiple of 4: padded leading dimension
    ld = -(-C // 4) * 4
    if kind == "constant": a = np.full((R, C), 3.25, np.float32)
    elif kind == "two_values": a = rng.choice(np.array([1.0, 2.0], np.float32), size=(R, C))
    elif kind == "tiny_range": a = (1.0 + 1e-6 * rng.random((R, C))).astype(np.float32)
    elif kind == "denormal": a = (1e-41 * rng.random((R, C))).astype(np.float32)
    elif kind == "negative": a = -np.abs(rng.standard_normal((R, C))).astype(np.float32)
    elif kind == "infinities":
        a = rng.standard_normal((R, C)).astype(np.float32)
        a[:, ::97] = np.inf
        a[:, 5::131] = -np.inf
    elif kind == "ascending": a = np.sort(rng.random((R, C)).astype(np.float32), axis=1)
    elif kind == "descending": a = -np.sort(-rng.random((R, C)).astype(np.float32), axis=1)
    elif kind == "spikes":
        a = np.zeros((R, C), np.float32)
        a[:, rng.integers(0, C, 50)] = rng.random(50).astype(np.float32)
    elif kind == "signed_zeros": a = rng.choice(np.array([0.0, -0.0, 1e-30, -1e-30], np.float32), size=(R, C))
    else: a = np.exp(3 * rng.standard_normal((R, C))).astype(np.float32)
    b = rng.standard_normal((R, C)).astype(np.float32)

    def padded(x):
        full = torch.zeros((R, ld), dtype=torch.float32, device=DEV)
        full[:, :C] = torch.from_numpy(x).to(DEV)
        return full[:, :C]

    cur, prev = padded(a), padded(b)
    for k in (1, 17, C // 14, C // 2, C - 1):
        for with_prev in (False, True):
            idx = torch.full((R, k), -1, dtype=torch.int32, device=DEV)
            counts = torch.zeros((R,), dtype=torch.int32, device=DEV)
            cm.topk_cols(cur, prev if with_prev else None, k, idx, counts)
            ref_idx, _ = oracle.topk_cols(a, b if with_prev else None, k)
            assert np.array_equal(idx.cpu().numpy(), ref_idx), (kind, k, with_prev)
            assert bool((counts == k).all())


# --------------------------------------------------------- bit-packed masks ---

@pytest.mark.parametrize("R,C,k", [
    (16, 1024, 256),          # Tiny attention rows
    (5, 1000, 1000),          # every column, C not a multiple of 32
    (7, 33, 5),
    (3, 1, 1),
    (24, 12288, 1229),        # FLUX MLP rows
    (6, 115456, 8082),        # HunyuanVideo attention rows: 3608 words per row
    (2, 1 << 20, 70000),      # the longest row indices_to_mask accepts
])
def test_mask_conversions_bit_exact(cm, oracle, R, C, k):
    """App. B.4 / Table 3: index lists -> bit-packed masks -> index lists, both kernels against the oracle, with
    different numbers of selected columns per row."""
    idx, counts = si.uniform_indices(R, C, k, 3, DEV, k_stride=k + 2)
    counts[0] = 0
    counts[R // 2] = max(1, k // 3)
    idx[:, k:] = -9                                                       # beyond the counts: never read
    words = -(-C // 32)
    ld = words + 1
    mask = torch.full((R, ld), -1, dtype=torch.int32, device=DEV)
    cm.indices_to_mask(idx, counts, C, mask)
    ref_mask = oracle.indices_to_mask(idx.cpu().numpy(), counts.cpu().numpy(), C, ld_words=ld, fill=0xffffffff)
    assert np.array_equal(mask.cpu().numpy().view(np.uint32), ref_mask)   # padding word untouched on both sides
    back = torch.full((R, k + 2), -7, dtype=torch.int32, device=DEV)
    back_counts = torch.full((R,), -7, dtype=torch.int32, device=DEV)
    cm.mask_to_indices(mask, C, back, back_counts)
    ref_idx, ref_counts = oracle.mask_to_indices(ref_mask, C, k + 2, idx_fill=-7)
    assert np.array_equal(back_counts.cpu().numpy(), ref_counts)
    assert np.array_equal(back.cpu().numpy(), ref_idx)
    assert np.array_equal(ref_counts, counts.cpu().numpy())               # the round trip returns the lists
    # a destination shorter than a row's population keeps the first columns
    short = torch.full((R, max(1, k // 2)), -7, dtype=torch.int32, device=DEV)
    cm.mask_to_indices(mask, C, short, back_counts)
    ref_idx, ref_counts = oracle.mask_to_indices(ref_mask, C, max(1, k // 2), idx_fill=-7)
    assert np.array_equal(short.cpu().numpy(), ref_idx) and np.array_equal(back_counts.cpu().numpy(), ref_counts)


def test_attention_from_bit_packed_masks_with_variable_counts(cm, oracle):
    """The memory-lean path: the pattern is kept as bit-packed masks whose rows select different numbers of
    columns; one conversion gives the lists and counts the delta kernel walks."""
    B, H, N, E, c = 1, 2, 900, 128, 192
    NB = -(-N // c)
    q, kk, v = recipes.attn_inputs(B, H, N, E, 8, DEV)
    g = si.generator(8, DEV)
    keep = torch.rand((B * H * NB, 1), generator=g, device=DEV) * 0.4            # 0 .. 40 % of the columns, per chunk
    dense = torch.rand((B * H * NB, N), generator=g, device=DEV) < keep
    dense[3] = False                                                             # one chunk selects nothing
    rows = torch.nonzero(dense)                                                  # the masks come from a list -> mask call
    k_stride = int(dense.sum(1).max())
    lists = torch.zeros((B * H * NB, k_stride), dtype=torch.int32, device=DEV)
    cnts = dense.sum(1).to(torch.int32)
    for r in range(B * H * NB):
        lists[r, :int(cnts[r])] = rows[rows[:, 0] == r, 1].to(torch.int32)
    mask = torch.zeros((B * H * NB, -(-N // 32)), dtype=torch.int32, device=DEV)
    cm.indices_to_mask(lists, cnts, N, mask)
    idx = torch.full((B * H * NB, k_stride), -1, dtype=torch.int32, device=DEV)
    counts = torch.zeros((B * H * NB,), dtype=torch.int32, device=DEV)
    cm.mask_to_indices(mask, N, idx, counts)
    assert torch.equal(counts, cnts) and int(counts.min()) == 0 and int(counts.max()) > int(counts.float().mean()) + 20
    base = recipes.attn_base((B, H, N, E), max(int(counts.float().mean()), 1), "delta", 8, DEV)
    out = torch.empty_like(base)
    scale = 1.0 / math.sqrt(E)
    cm.attn_sparse_delta(q, kk, v, idx.view(B, H, NB, -1), counts.view(B, H, NB), base, out, c, scale, 1.0)
    basen = si.np_f32(base).astype(np.float64)
    ref = oracle.attn_sparse_delta(si.np_f32(q), si.np_f32(kk), si.np_f32(v), idx.cpu().numpy().reshape(B, H, NB, -1),
                                   counts.cpu().numpy().reshape(B, H, NB), basen, c, scale, 1.0)
    assert rel_err(si.np_f32(out), ref, ref - basen) <= REL_TOL


# ---------------------------------------------------------------- attention ---

def _attn_case(B, H, N, E, c, k, seed, ragged, order="ascending", base_mode="unit"):
    q, kk, v = recipes.attn_inputs(B, H, N, E, seed, DEV)
    NB = -(-N // c)
    idx, counts = recipes.attn_indices(B * H * NB, N, k, seed, DEV, ragged, order)
    idx = idx.view(B, H, NB, k).contiguous()
    counts = counts.view(B, H, NB).contiguous()
    base = recipes.attn_base((B, H, N, E), k, base_mode, seed, DEV)
    return q, kk, v, idx, counts, base


@pytest.mark.parametrize("B,H,N,E,c,k,ragged", [
    (1, 2, 1024, 64, 128, 256, False),     # Tiny (config 0)
    (1, 2, 1000, 64, 128, 250, True),      # ragged last chunk, ragged counts
    (1, 2, 1100, 128, 192, 100, True),
    (2, 3, 700, 128, 128, 333, True),
    (1, 1, 500, 64, 192, 77, True),
    (1, 1, 192, 128, 192, 192, False),     # one chunk, every column
    (1, 1, 50, 128, 192, 7, False),        # fewer rows than one MFMA tile group
])
def test_attn_sparse_delta_parity(cm, oracle, B, H, N, E, c, k, ragged):
    q, kk, v, idx, counts, base = _attn_case(B, H, N, E, c, k, 0, ragged)
    scale = 1.0 / math.sqrt(E)
    qn, kn, vn = si.np_f32(q), si.np_f32(kk), si.np_f32(v)
    basen = si.np_f32(base).astype(np.float64)
    idxn, cntn = idx.cpu().numpy(), counts.cpu().numpy()
    for o_scale in (1.0, -1.0):
        out = torch.empty_like(base)
        cm.attn_sparse_delta(q, kk, v, idx, counts, base, out, c, scale, o_scale)
        ref = oracle.attn_sparse_delta(qn, kn, vn, idxn, cntn, basen, c, scale, o_scale)
        assert rel_err(si.np_f32(out), ref, ref - basen) <= REL_TOL
    # counts == 0 units return the cache bit for bit
    zero_units = np.argwhere(cntn == 0)
    for b, h, i in zero_units:
        assert torch.equal(out[b, h, i * c:(i + 1) * c], base[b, h, i * c:(i + 1) * c])
    # in place: out aliases base
    inplace = base.clone()
    cm.attn_sparse_delta(q, kk, v, idx, counts, inplace, inplace, c, scale, -1.0)
    assert torch.equal(inplace, out)


@pytest.mark.parametrize("order", ["shuffled", "duplicates"])
@pytest.mark.parametrize("B,H,N,E,c,k", [(1, 2, 700, 128, 192, 100), (1, 2, 1024, 64, 128, 77)])
def test_attn_index_list_is_taken_as_given(cm, oracle, order, B, H, N, E, c, k):
    """Alg. 3 walks the list it is handed: an unsorted list gives the sorted list's result, and a column listed
    twice counts twice in the softmax (the list is a multiset).  Cache at the delta's own scale."""
    q, kk, v, idx, counts, base = _attn_case(B, H, N, E, c, k, 21, True, order, "delta")
    scale = 1.0 / math.sqrt(E)
    basen = si.np_f32(base).astype(np.float64)
    out = torch.empty_like(base)
    cm.attn_sparse_delta(q, kk, v, idx, counts, base, out, c, scale, 1.0)
    ref = oracle.attn_sparse_delta(si.np_f32(q), si.np_f32(kk), si.np_f32(v), idx.cpu().numpy(), counts.cpu().numpy(),
                                   basen, c, scale, 1.0)
    assert rel_err(si.np_f32(out), ref, ref - basen) <= REL_TOL
    if order == "duplicates":     # the multiset matters: the deduplicated list gives a different answer
        flat_i, flat_c = idx.view(-1, k).cpu().numpy(), counts.view(-1).cpu().numpy()
        assert any(len(set(flat_i[u, :flat_c[u]])) < flat_c[u] for u in range(len(flat_c)))


@pytest.mark.parametrize("B,H,N,E,c,n_blocks,ragged", [
    (1, 2, 1024, 64, 128, 2, False),       # Tiny: 2 of 8 blocks
    (1, 2, 1100, 128, 192, 3, True),       # the sequence's last block holds 76 columns; ragged last chunk
    (2, 2, 700, 128, 128, 2, True),
    (1, 1, 500, 64, 192, 4, True),         # every block (N < 4 * 128): dense, with the partial block
    (1, 1, 100, 128, 192, 1, False),       # one partial block
])
def test_attn_block_sparse_delta_parity(cm, oracle, B, H, N, E, c, n_blocks, ragged):
    """The [c, 128] block pattern of Table 2: the kernel that walks a list of 128-column key blocks against the
    oracle's Alg. 3 on the list of all columns of those blocks."""
    q, kk, v = recipes.attn_inputs(B, H, N, E, 4, DEV)
    NB = -(-N // c)
    units = B * H * NB
    blocks, bcounts = recipes.attn_block_lists(units, N, n_blocks, 4, DEV, ragged)
    idxn, cntn = recipes.expand_block_lists(blocks.cpu().numpy(), bcounts.cpu().numpy(), N)
    k_kept = max(int(cntn.max()), 1)
    base = recipes.attn_base((B, H, N, E), k_kept, "delta", 4, DEV)
    basen = si.np_f32(base).astype(np.float64)
    scale = 1.0 / math.sqrt(E)
    blocks4 = blocks.view(B, H, NB, n_blocks).contiguous()
    bcounts3 = bcounts.view(B, H, NB).contiguous()
    for o_scale in (1.0, -1.0):
        out = torch.full_like(base, float("nan"))
        cm.attn_block_sparse_delta(q, kk, v, blocks4, bcounts3, base, out, c, scale, o_scale)
        ref = oracle.attn_sparse_delta(si.np_f32(q), si.np_f32(kk), si.np_f32(v), idxn.reshape(B, H, NB, -1),
                                       cntn.reshape(B, H, NB), basen, c, scale, o_scale)
        assert rel_err(si.np_f32(out), ref, ref - basen) <= REL_TOL
    for b, h, i in np.argwhere(cntn.reshape(B, H, NB) == 0):       # nothing selected: the cache, bit for bit
        assert torch.equal(out[b, h, i * c:(i + 1) * c], base[b, h, i * c:(i + 1) * c])
    # the column-list kernel on the expanded lists gives the same result up to the order of the accumulation
    idx_t = torch.from_numpy(idxn).to(DEV).view(B, H, NB, -1).contiguous()
    cnt_t = torch.from_numpy(cntn).to(DEV).view(B, H, NB).contiguous()
    out_cols = torch.empty_like(base)
    cm.attn_sparse_delta(q, kk, v, idx_t, cnt_t, base, out_cols, c, scale, -1.0)
    assert rel_err(si.np_f32(out_cols), si.np_f32(out).astype(np.float64), ref - basen) <= 1e-2


def test_attn_block_sparse_hunyuan_shape_sampled_units(cm, oracle):
    """The launch bench.py times for the block pattern (63 of 902 blocks per chunk, the kept count of 93 %
    sparsity), sampled units against the oracle on a zero cache and on a cache at the delta's scale."""
    cfg = si.CONFIGS["hunyuan"]
    B, H, E, c = cfg["B"], cfg["H"], cfg["E"], cfg["c"]
    N = si.config_tokens(cfg)
    NB = -(-N // c)
    n_blocks = si.kept(N, cfg["attn_keep"]) // cm.ATTN_BLOCK_COLUMNS
    q, kk, v = recipes.attn_inputs(B, H, N, E, 0, DEV)
    blocks, bcounts = recipes.attn_block_lists(B * H * NB, N, n_blocks, 0, DEV)
    blocks4, bcounts3 = blocks.view(B, H, NB, n_blocks), bcounts.view(B, H, NB)
    scale = 1.0 / math.sqrt(E)
    rng = np.random.default_rng(1)
    units = [(0, 0, 0), (B - 1, H - 1, NB - 1)] + [(int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(NB)))
                                                     for _ in range(3)]
    for mode in ("zero", "delta"):
        base = recipes.attn_base((B, H, N, E), n_blocks * cm.ATTN_BLOCK_COLUMNS, mode, 0, DEV)
        out = torch.empty_like(base)
        cm.attn_block_sparse_delta(q, kk, v, blocks4, bcounts3, base, out, c, scale, 1.0)
        torch.cuda.synchronize()
        for b, h, i in units:
            rows = slice(i * c, min(N, (i + 1) * c))
            idxn, cntn = recipes.expand_block_lists(blocks4[b, h, i:i + 1].cpu().numpy(), bcounts3[b, h, i:i + 1].cpu().numpy(), N)
            basen = si.np_f32(base[b:b + 1, h:h + 1, rows]).astype(np.float64)
            ref = oracle.attn_sparse_delta(si.np_f32(q[b:b + 1, h:h + 1, rows]), si.np_f32(kk[b:b + 1, h:h + 1]),
                                           si.np_f32(v[b:b + 1, h:h + 1]), idxn.reshape(1, 1, 1, -1), cntn.reshape(1, 1, 1),
                                           basen, c, scale, 1.0)
            assert rel_err(si.np_f32(out[b:b + 1, h:h + 1, rows]), ref, ref - basen) <= REL_TOL, (mode, b, h, i)
        del base, out


def test_attn_all_columns_equals_dense_and_cache_roundtrip(cm, oracle):
    """k = N reproduces dense attention; O_cache = O - Delta then O_cache + Delta returns O (Alg. 2)."""
    B, H, N, E, c = 1, 2, 520, 128, 192
    q, kk, v, idx, counts, _ = _attn_case(B, H, N, E, c, 60, 3, False)
    scale = 1.0 / math.sqrt(E)
    dense = torch.empty_like(q)
    cm.attn_sparse_delta(q, kk, v, None, None, None, dense, c, scale, 1.0)
    ref = oracle.attn_dense(si.np_f32(q), si.np_f32(kk), si.np_f32(v), c, scale)
    assert rel_err(si.np_f32(dense), ref) <= REL_TOL
    # each call is compared with the oracle applied to the call's own bf16 input cache
    qn, kn, vn = si.np_f32(q), si.np_f32(kk), si.np_f32(v)
    idxn, cntn = idx.cpu().numpy(), counts.cpu().numpy()
    dense_n = si.np_f32(dense).astype(np.float64)
    cache = torch.empty_like(q)
    cm.attn_sparse_delta(q, kk, v, idx, counts, dense, cache, c, scale, -1.0)
    cache_ref = oracle.attn_sparse_delta(qn, kn, vn, idxn, cntn, dense_n, c, scale, -1.0)
    assert rel_err(si.np_f32(cache), cache_ref, cache_ref - dense_n) <= REL_TOL
    again = torch.empty_like(q)
    cm.attn_sparse_delta(q, kk, v, idx, counts, cache, again, c, scale, 1.0)
    cache_n = si.np_f32(cache).astype(np.float64)
    again_ref = oracle.attn_sparse_delta(qn, kn, vn, idxn, cntn, cache_n, c, scale, 1.0)
    # Here the cache and the delta are each about three times larger than their sum (60 of 520 columns carry a
    # softmax of their own), so the sum cancels: the update's RMS is the floor of the metric.
    assert rel_err(si.np_f32(again), again_ref, again_ref - cache_n) <= REL_TOL
    # the round trip returns the dense output up to the bf16 rounding of the stored cache, whose
    # entries (dense minus delta) are larger than the dense output's: 2^-8 of the cache's largest entry
    bound = float(np.abs(cache_ref).max()) * 2.0 ** -8 + REL_TOL * float(np.sqrt(np.mean(ref * ref)))
    assert float(np.abs(si.np_f32(again) - ref).max()) <= bound


@pytest.mark.parametrize("B,H,N,E,c", [(1, 2, 1024, 64, 128), (1, 2, 700, 128, 192), (1, 2, 520, 64, 192),
                                       (2, 1, 600, 128, 128)])   # the four instantiations of the every-column mode
def test_attn_dense_with_colsum_parity(cm, oracle, B, H, N, E, c):
    (q, kk, v), _, _ = si.attn_steps(B, H, N, E, 5, DEV)
    scale = 1.0 / math.sqrt(E)
    NB = -(-N // c)
    ld = -(-N // 4) * 4
    out = torch.empty_like(q)
    D = torch.full((B, H, NB, ld), -1.0, dtype=torch.float32, device=DEV)
    ws = _u8(cm.attn_dense_workspace_bytes(B, H, N))
    cm.attn_dense(q, kk, v, out, D, c, scale, ws)
    ref, Dref = oracle.attn_dense(si.np_f32(q), si.np_f32(kk), si.np_f32(v), c, scale, want_colsum=True)
    assert rel_err(si.np_f32(out), ref) <= REL_TOL
    Dg = D.cpu().numpy()[..., :N].astype(np.float64)
    assert rel_err(Dg, Dref) <= REL_TOL
    rows = np.array([min(c, N - i * c) for i in range(NB)], np.float64)
    assert np.allclose(Dg.sum(-1), rows[None, None], rtol=2e-3)     # each row of P sums to one


@pytest.mark.parametrize("B,H,N,E,c", [(1, 2, 1024, 64, 128), (2, 2, 700, 128, 192)])
def test_attn_colsum_with_stale_normalisers_parity(cm, oracle, B, H, N, E, c):
    """Alg. 4: the dense pass of one step leaves (m, l); the next step's column sums are taken against them."""
    (q1, k1, v1), (q2, k2, _), _ = si.attn_steps(B, H, N, E, 7, DEV)
    scale = 1.0 / math.sqrt(E)
    NB = -(-N // c)
    ld = -(-N // 4) * 4
    out = torch.empty_like(q1)
    D1 = torch.empty((B, H, NB, ld), dtype=torch.float32, device=DEV)
    ws = _u8(cm.attn_dense_workspace_bytes(B, H, N))
    cm.attn_dense(q1, k1, v1, out, D1, c, scale, ws)
    m, l = cm.attn_dense_row_stats(ws, B, H, N)
    m, l = m.clone(), l.clone()
    # the statistics are a valid (reference, sum) pair: m + log l is the row's log-sum-exp, whatever reference m is
    m_ref, l_ref = oracle.attn_row_stats(si.np_f32(q1), si.np_f32(k1), scale)
    lse = m.cpu().numpy().astype(np.float64) + np.log(l.cpu().numpy().astype(np.float64))
    assert np.abs(lse - (m_ref + np.log(l_ref))).max() <= 2e-3
    assert (m.cpu().numpy() <= m_ref + 1e-3).all()        # a reference no larger than the row maximum ...
    assert (m.cpu().numpy() >= m_ref - 8 * math.log(2.0) - 1e-3).all()   # ... and within 2^8 of it
    # same step, same statistics: the exact column sums again
    D_same = torch.full((B, H, NB, ld), -1.0, dtype=torch.float32, device=DEV)
    cm.attn_colsum_stale(q1, k1, m, l, D_same, c, scale)
    assert rel_err(D_same.cpu().numpy()[..., :N], D1.cpu().numpy()[..., :N].astype(np.float64)) <= 1e-4
    # next step against the stale statistics
    D2 = torch.full((B, H, NB, ld), -1.0, dtype=torch.float32, device=DEV)
    cm.attn_colsum_stale(q2, k2, m, l, D2, c, scale)
    ref = oracle.attn_colsum_stale(si.np_f32(q2), si.np_f32(k2), m.cpu().numpy().astype(np.float64),
                                   l.cpu().numpy().astype(np.float64), c, scale)
    got = D2.cpu().numpy()
    assert rel_err(got[..., :N].astype(np.float64), ref) <= REL_TOL
    assert (got[..., N:] == -1.0).all()                   # padding columns are not written
    # and the selection it feeds (Alg. 4 -> top-k) is almost the one the exact column sums give
    exact = oracle.attn_dense(si.np_f32(q2), si.np_f32(k2), si.np_f32(v1), c, scale, want_colsum=True)[1]
    kk = max(8, N // 8)
    top_stale = np.argsort(-got[..., :N], axis=-1)[..., :kk]
    top_exact = np.argsort(-exact, axis=-1)[..., :kk]
    overlap = np.mean([len(set(a) & set(b)) / kk for a, b in zip(top_stale.reshape(-1, kk), top_exact.reshape(-1, kk))])
    assert overlap >= 0.9      # the approximation App. B.2 relies on: stale normalisers barely move the top-k set


@pytest.mark.parametrize("B,H,N,E,c", [(1, 2, 1024, 64, 128), (2, 2, 700, 128, 192), (1, 1, 100, 128, 128),
                                       (1, 2, 333, 64, 192), (1, 1, 1, 128, 192)])
def test_attn_dense_fused_with_stale_column_sums_parity(cm, oracle, B, H, N, E, c):
    """Alg. 4 in one kernel: dense output, column sums against the previous step's normalisers, and this step's
    normalisers for the next one."""
    (q1, k1, v1), (q2, k2, v2), _ = si.attn_steps(B, H, N, E, 11, DEV)
    scale = 1.0 / math.sqrt(E)
    NB = -(-N // c)
    ld = -(-N // 4) * 4
    out1 = torch.empty_like(q1)
    D1 = torch.empty((B, H, NB, ld), dtype=torch.float32, device=DEV)
    ws = _u8(cm.attn_dense_workspace_bytes(B, H, N))
    cm.attn_dense(q1, k1, v1, out1, D1, c, scale, ws)                    # step 1: leaves (m, l)
    m1, l1 = (t.clone() for t in cm.attn_dense_row_stats(ws, B, H, N))
    out2 = torch.empty_like(q2)
    D2 = torch.full((B, H, NB, ld), -1.0, dtype=torch.float32, device=DEV)
    m2 = torch.empty_like(m1)
    l2 = torch.empty_like(l1)
    cm.attn_dense_colsum_stale(q2, k2, v2, out2, m1, l1, D2, c, scale, m2, l2)   # step 2
    qn, kn, vn = si.np_f32(q2), si.np_f32(k2), si.np_f32(v2)
    assert rel_err(si.np_f32(out2), oracle.attn_dense(qn, kn, vn, c, scale)) <= REL_TOL
    ref = oracle.attn_colsum_stale(qn, kn, m1.cpu().numpy().astype(np.float64), l1.cpu().numpy().astype(np.float64), c, scale)
    got = D2.cpu().numpy()
    assert rel_err(got[..., :N].astype(np.float64), ref) <= REL_TOL
    assert (got[..., N:] == -1.0).all()
    m_ref, l_ref = oracle.attn_row_stats(qn, kn, scale)
    lse = m2.cpu().numpy().astype(np.float64) + np.log(l2.cpu().numpy().astype(np.float64))
    assert np.abs(lse - (m_ref + np.log(l_ref))).max() <= 2e-3
    # the separate pass over the same inputs gives the same sums
    D2b = torch.empty_like(D2)
    cm.attn_colsum_stale(q2, k2, m1, l1, D2b, c, scale)
    assert rel_err(got[..., :N].astype(np.float64), D2b.cpu().numpy()[..., :N].astype(np.float64)) <= 1e-3
    # without the statistics outputs
    out3 = torch.empty_like(q2)
    D3 = torch.empty_like(D2)
    cm.attn_dense_colsum_stale(q2, k2, v2, out3, m1, l1, D3, c, scale)
    assert torch.equal(out3, out2) and torch.equal(D3[..., :N], D2[..., :N])


@pytest.mark.parametrize("B,H,N,E,c", [(1, 2, 700, 128, 192), (1, 1, 300, 64, 128)])
def test_attn_column_sums_with_far_stale_normalisers(cm, oracle, B, H, N, E, c):
    """Normalisers far below the current scores.  60 below: every weight is near e^60, inside fp32, and both
    entry points still evaluate Alg. 4's expression.  200 below: every weight is beyond fp32; the separate pass
    overflows to +inf like the expression, the fused kernel saturates to a large number or +inf, neither to NaN."""
    (q1, k1, v1), (q2, k2, v2), _ = si.attn_steps(B, H, N, E, 13, DEV)
    scale = 1.0 / math.sqrt(E)
    NB = -(-N // c)
    ld = -(-N // 4) * 4
    out = torch.empty_like(q1)
    D1 = torch.empty((B, H, NB, ld), dtype=torch.float32, device=DEV)
    ws = _u8(cm.attn_dense_workspace_bytes(B, H, N))
    cm.attn_dense(q1, k1, v1, out, D1, c, scale, ws)
    m1, l1 = (t.clone() for t in cm.attn_dense_row_stats(ws, B, H, N))
    qn, kn = si.np_f32(q2), si.np_f32(k2)
    m_far = m1 - 60.0
    ref = oracle.attn_colsum_stale(qn, kn, m_far.cpu().numpy().astype(np.float64), l1.cpu().numpy().astype(np.float64),
                                   c, scale)
    D_fused = torch.empty_like(D1)
    cm.attn_dense_colsum_stale(q2, k2, v2, out, m_far, l1, D_fused, c, scale)
    D_pass = torch.empty_like(D1)
    cm.attn_colsum_stale(q2, k2, m_far, l1, D_pass, c, scale)
    assert rel_err(D_fused.cpu().numpy()[..., :N].astype(np.float64), ref) <= REL_TOL
    assert rel_err(D_pass.cpu().numpy()[..., :N].astype(np.float64), ref) <= REL_TOL
    m_gone = m1 - 200.0
    cm.attn_dense_colsum_stale(q2, k2, v2, out, m_gone, l1, D_fused, c, scale)
    cm.attn_colsum_stale(q2, k2, m_gone, l1, D_pass, c, scale)
    fused, alone = D_fused[..., :N], D_pass[..., :N]
    assert not bool(torch.isnan(fused).any()) and not bool(torch.isnan(alone).any())
    assert bool((fused >= 2.0 ** 100).all()) and bool(torch.isinf(alone).all())
    # the attention output itself does not depend on the stale normalisers
    assert rel_err(si.np_f32(out), oracle.attn_dense(qn, kn, si.np_f32(v2), c, scale)) <= REL_TOL


def _check_sampled_attn_units(cm, oracle, name, n_units, sparse_k):
    """Full-shape launch, sampled (batch, head, chunk) units against the oracle.  Run twice: on a zero cache (the
    output IS the delta) and on a cache drawn at the delta's own scale, so that nothing hides a wrong delta."""
    cfg = si.CONFIGS[name]
    B, H, E, c = cfg["B"], cfg["H"], cfg["E"], cfg["c"]
    N = si.config_tokens(cfg)
    q, kk, v = recipes.attn_inputs(B, H, N, E, 0, DEV)
    NB = -(-N // c)
    idx, counts = recipes.attn_indices(B * H * NB, N, sparse_k, 0, DEV)
    idx = idx.view(B, H, NB, sparse_k)
    counts = counts.view(B, H, NB)
    scale = 1.0 / math.sqrt(E)
    rng = np.random.default_rng(0)
    units = [(0, 0, 0), (B - 1, H - 1, NB - 1)] + [(int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(NB)))
                                                     for _ in range(n_units - 2)]
    for mode in ("zero", "delta"):
        base = recipes.attn_base((B, H, N, E), sparse_k, mode, 0, DEV)
        out = torch.empty_like(base)
        cm.attn_sparse_delta(q, kk, v, idx, counts, base, out, c, scale, 1.0)
        torch.cuda.synchronize()
        worst = 0.0
        for b, h, i in units:
            rows = slice(i * c, min(N, (i + 1) * c))
            basen = si.np_f32(base[b:b + 1, h:h + 1, rows]).astype(np.float64)
            ref = oracle.attn_sparse_delta(si.np_f32(q[b:b + 1, h:h + 1, rows]), si.np_f32(kk[b:b + 1, h:h + 1]),
                                           si.np_f32(v[b:b + 1, h:h + 1]),
                                           np.ascontiguousarray(idx[b:b + 1, h:h + 1, i:i + 1].cpu().numpy()),
                                           np.ascontiguousarray(counts[b:b + 1, h:h + 1, i:i + 1].cpu().numpy()),
                                           basen, c, scale, 1.0)
            worst = max(worst, rel_err(si.np_f32(out[b:b + 1, h:h + 1, rows]), ref, ref - basen))
        assert worst <= REL_TOL, mode
        del base, out


def test_attn_flux_shape_sampled_units(cm, oracle):
    _check_sampled_attn_units(cm, oracle, "flux", 12, 323)


def test_attn_hunyuan_shape_sampled_units(cm, oracle):
    _check_sampled_attn_units(cm, oracle, "hunyuan", 6, 8082)


def test_attn_wan_shape_sampled_units(cm, oracle):
    _check_sampled_attn_units(cm, oracle, "wan", 6, 5292)


def test_attn_dense_and_column_sums_hunyuan_shape_sampled_units(cm, oracle):
    """The dense step at the full HunyuanVideo shape (the launch bench.py uses to fill the caches): output, exact
    column sums and the stale-normaliser column sums (as a pass of their own and from the attention kernel) of
    sampled chunks against the oracle."""
    cfg = si.CONFIGS["hunyuan"]
    B, H, E, c = cfg["B"], cfg["H"], cfg["E"], cfg["c"]
    N = si.config_tokens(cfg)
    (q1, k1, v1), (q2, k2, _), _ = si.attn_steps(B, H, N, E, 3, DEV)
    del v1
    v = si.randn_bf16((B, H, N, E), si.generator(4, DEV))
    NB = -(-N // c)
    ld = -(-N // 4) * 4
    scale = 1.0 / math.sqrt(E)
    out = torch.empty_like(q1)
    D = torch.empty((B, H, NB, ld), dtype=torch.float32, device=DEV)
    ws = _u8(cm.attn_dense_workspace_bytes(B, H, N))
    cm.attn_dense(q1, k1, v, out, D, c, scale, ws)
    m, l = cm.attn_dense_row_stats(ws, B, H, N)
    D2 = torch.empty_like(D)
    cm.attn_colsum_stale(q2, k2, m, l, D2, c, scale)
    out3 = torch.empty_like(q2)
    D3 = torch.empty_like(D)
    m3, l3 = torch.empty_like(m), torch.empty_like(l)
    cm.attn_dense_colsum_stale(q2, k2, v, out3, m, l, D3, c, scale, m3, l3)
    torch.cuda.synchronize()
    for b, h, i in [(0, 0, 0), (B - 1, H - 1, NB - 1), (0, H // 2, NB // 3)]:
        rows = slice(i * c, min(N, (i + 1) * c))
        kn, vn = si.np_f32(k1[b:b + 1, h:h + 1]), si.np_f32(v[b:b + 1, h:h + 1])
        ref, Dref = oracle.attn_dense(si.np_f32(q1[b:b + 1, h:h + 1, rows]), kn, vn, c, scale, want_colsum=True)
        assert rel_err(si.np_f32(out[b:b + 1, h:h + 1, rows]), ref) <= REL_TOL, (b, h, i)
        assert rel_err(D[b, h, i, :N].cpu().numpy().astype(np.float64), Dref[0, 0, 0]) <= REL_TOL, (b, h, i)
        ms = m[b:b + 1, h:h + 1, rows].cpu().numpy().astype(np.float64)
        ls = l[b:b + 1, h:h + 1, rows].cpu().numpy().astype(np.float64)
        ref2 = oracle.attn_colsum_stale(si.np_f32(q2[b:b + 1, h:h + 1, rows]), si.np_f32(k2[b:b + 1, h:h + 1]), ms, ls, c,
                                        scale)
        assert rel_err(D2[b, h, i, :N].cpu().numpy().astype(np.float64), ref2[0, 0, 0]) <= REL_TOL, (b, h, i)
        assert rel_err(D3[b, h, i, :N].cpu().numpy().astype(np.float64), ref2[0, 0, 0]) <= REL_TOL, (b, h, i)
        q2n, k2n = si.np_f32(q2[b:b + 1, h:h + 1, rows]), si.np_f32(k2[b:b + 1, h:h + 1])
        assert rel_err(si.np_f32(out3[b:b + 1, h:h + 1, rows]), oracle.attn_dense(q2n, k2n, vn, c, scale)) <= REL_TOL
        m_ref, l_ref = oracle.attn_row_stats(q2n, k2n, scale)
        lse = (m3[b, h, rows].cpu().numpy().astype(np.float64) + np.log(l3[b, h, rows].cpu().numpy().astype(np.float64)))
        assert np.abs(lse - (m_ref + np.log(l_ref))[0, 0]).max() <= 2e-3, (b, h, i)


# ---------------------------------------------------------------------- MLP ---

@pytest.mark.parametrize("B,N,D,F,c,act", [
    (1, 1024, 256, 1024, 128, 1),          # Tiny (config 0)
    (2, 500, 256, 320, 192, 0),            # ragged last chunk, erf GELU, F not a multiple of 128
    (1, 200, 128, 64, 128, 1),
])
def test_mlp_dense_and_tile_mean_parity(cm, oracle, B, N, D, F, c, act):
    x1, _, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 0, DEV)
    a_ld = -(-N // 8) * 8 + 8
    out = torch.empty_like(x1)
    a_cache = torch.zeros((B, F, a_ld), dtype=torch.bfloat16, device=DEV)
    cm.mlp_dense(x1, w1, b1, w2, b2, out, a_cache, c, act)
    ref, a_ref, T_ref = oracle.mlp_dense(si.np_f32(x1), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), si.np_f32(b2),
                                         c, act, a_ld=a_ld)
    assert rel_err(si.np_f32(a_cache)[..., :N], a_ref[..., :N]) <= REL_TOL
    assert torch.all(a_cache[..., N:] == 0)                          # padding of the cache rows untouched
    assert rel_err(si.np_f32(out), ref) <= REL_TOL
    NB = -(-N // c)
    T = torch.empty((B, NB, F), dtype=torch.float32, device=DEV)
    ws = _u8(cm.mlp_tile_mean_workspace_bytes(B, N, D, F, c))
    cm.mlp_tile_mean_preact(x1, w1, T, c, ws)
    assert rel_err(T.cpu().numpy(), T_ref) <= SCORE_TOL              # split-precision mean: far tighter than bf16
    assert rel_err(T.cpu().numpy(), oracle.mlp_tile_scores(si.np_f32(x1), si.np_f32(w1), c)) <= SCORE_TOL


@pytest.mark.parametrize("B,N,D,F,c", [
    (1, 200 * 128, 128, 64, 128),          # 200 chunks: two row blocks of the scores GEMM, the second one ragged
    (2, 150 * 192 - 50, 256, 320, 192),    # 300 chunks over two batches, ragged last chunk, F not a multiple of 128
])
def test_mlp_tile_mean_many_chunks(cm, oracle, B, N, D, F, c):
    """Token-merged pre-activations (Alg. 7) with more chunks than one 128-row block of the scores GEMM holds:
    the path the video shapes take (602 and 394 chunks)."""
    g = si.generator(5, DEV)
    x = si.randn_bf16((B, N, D), g)
    w1 = si.randn_bf16((F, D), g, 1.0 / math.sqrt(D))
    NB = -(-N // c)
    assert B * NB > 128
    T = torch.full((B, NB, F), float("nan"), dtype=torch.float32, device=DEV)
    cm.mlp_tile_mean_preact(x, w1, T, c, _u8(cm.mlp_tile_mean_workspace_bytes(B, N, D, F, c)))
    assert rel_err(T.cpu().numpy(), oracle.mlp_tile_scores(si.np_f32(x), si.np_f32(w1), c)) <= SCORE_TOL


@pytest.mark.parametrize("name", ["hunyuan", "wan"])
def test_mlp_tile_mean_full_shape_sampled_chunks(cm, oracle, name):
    """The scores launch bench.py times (five / four row blocks, the contraction cut in two pieces): sampled
    chunks' rows of T against the oracle, each chunk a B = 1, N = rows problem."""
    cfg = si.CONFIGS[name]
    B, D, F, c = cfg["B"], cfg["D"], cfg["F"], cfg["c"]
    N = si.config_tokens(cfg)
    NB = -(-N // c)
    g = si.generator(6, DEV)
    x = si.randn_bf16((B, N, D), g)
    w1 = si.randn_bf16((F, D), g, 1.0 / math.sqrt(D))
    T = torch.full((B, NB, F), float("nan"), dtype=torch.float32, device=DEV)
    cm.mlp_tile_mean_preact(x, w1, T, c, _u8(cm.mlp_tile_mean_workspace_bytes(B, N, D, F, c)))
    torch.cuda.synchronize()
    assert bool(torch.isfinite(T).all())
    w1n = si.np_f32(w1)
    for i in (0, 127, 128, 300, NB - 2, NB - 1):                     # both sides of a row-block edge, the ragged last chunk
        rows = slice(i * c, min(N, (i + 1) * c))
        ref = oracle.mlp_tile_scores(si.np_f32(x[:, rows]), w1n, c)
        assert rel_err(T[:, i:i + 1].cpu().numpy(), ref) <= SCORE_TOL, i


@pytest.mark.parametrize("B,N,D,F,c,k,act", [
    (1, 1024, 256, 1024, 128, 256, 1),     # Tiny (config 0)
    (2, 500, 256, 320, 192, 100, 0),       # ragged chunk, counts not multiples of the tiles
    (1, 300, 128, 256, 128, 256, 1),       # every neuron selected
    (1, 192, 128, 128, 192, 1, 1),         # one neuron
])
def test_mlp_sparse_delta_parity(cm, oracle, B, N, D, F, c, k, act):
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 1, DEV)
    a_ld = -(-N // 8) * 8
    NB = -(-N // c)
    # caches of the dense step, from the oracle, rounded to the bf16 storage format
    o_ref, a_ref, _ = oracle.mlp_dense(si.np_f32(x1), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), si.np_f32(b2),
                                       c, act, a_ld=a_ld)
    o_cache = torch.from_numpy(o_ref).to(torch.bfloat16).to(DEV)
    a_cache = torch.from_numpy(a_ref).to(torch.bfloat16).to(DEV)
    o_ref = si.np_f32(o_cache).astype(np.float64)
    a_ref = si.np_f32(a_cache).astype(np.float64)
    ws = _u8(cm.mlp_workspace_bytes(B, N, D, F, c, k))
    for step in range(2):                                            # two sparse steps in a row on the same caches
        idx, counts = recipes.mlp_indices(B * NB, F, k, 10 + step, DEV, ragged=True)
        idx = idx.view(B, NB, k).contiguous()
        counts = counts.view(B, NB).contiguous()
        a_before = a_cache.clone()
        o_before = o_ref.copy()                                      # the oracle's caches are chained over both steps
        cm.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, a_cache, o_cache, c, act, ws)
        oracle.mlp_sparse_delta(si.np_f32(x2), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), idx.cpu().numpy(),
                                counts.cpu().numpy(), a_ref, o_ref, c, act)
        assert rel_err(si.np_f32(a_cache)[..., :N], a_ref[..., :N]) <= REL_TOL
        assert rel_err(si.np_f32(o_cache), o_ref, o_ref - o_before) <= REL_TOL
        # unselected cells of a_cache are untouched, bit for bit
        touched = torch.zeros((B, F, a_ld), dtype=torch.bool, device=DEV)
        for b in range(B):
            for i in range(NB):
                sel = idx[b, i, :int(counts[b, i])].long()
                touched[b, sel, i * c:min(N, (i + 1) * c)] = True
        assert torch.equal(a_cache[~touched], a_before[~touched])
        x2 = si.randn_bf16(tuple(x2.shape), si.generator(77 + step, DEV))


@pytest.mark.parametrize("name,chunks", [("flux", (0, 7, -1)), ("hunyuan", (0, -1)), ("wan", (3, -1))])
def test_mlp_full_shape_sampled_units(cm, oracle, name, chunks):
    cfg = si.CONFIGS[name]
    B, D, F, c = cfg["B"], cfg["D"], cfg["F"], cfg["c"]
    N = si.config_tokens(cfg)
    k = si.kept(F, cfg["mlp_keep"])
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 2, DEV)
    NB = -(-N // c)
    act = 1
    out = torch.empty_like(x1)
    a_cache = torch.zeros((B, F, N), dtype=torch.bfloat16, device=DEV)
    cm.mlp_dense(x1, w1, b1, w2, b2, out, a_cache, c, act)
    idx, counts = recipes.mlp_indices(B * NB, F, k, 3, DEV)
    idx = idx.view(B, NB, k).contiguous()
    counts = counts.view(B, NB).contiguous()
    a0, o0 = a_cache.clone(), out.clone()
    ws = _u8(cm.mlp_workspace_bytes(B, N, D, F, c, k))
    cm.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, a_cache, out, c, act, ws)
    torch.cuda.synchronize()
    w1n, b1n, w2n, b2n = si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), si.np_f32(b2)
    for i in [ch % NB for ch in chunks]:                              # sampled token chunks, each a B=1, N=c problem
        rows = slice(i * c, min(N, (i + 1) * c))
        dref = oracle.mlp_dense(si.np_f32(x1[:, rows]), w1n, b1n, w2n, b2n, c, act, want_caches=False)
        assert rel_err(si.np_f32(o0[:, rows]), dref) <= REL_TOL       # dense kernel at this shape
        a_u = np.ascontiguousarray(si.np_f32(a0[:, :, rows]).astype(np.float64))
        o_before = np.ascontiguousarray(si.np_f32(o0[:, rows]).astype(np.float64))
        o_u = o_before.copy()
        oracle.mlp_sparse_delta(si.np_f32(x2[:, rows]), w1n, b1n, w2n, np.ascontiguousarray(idx[:, i:i + 1].cpu().numpy()),
                                np.ascontiguousarray(counts[:, i:i + 1].cpu().numpy()), a_u, o_u, c, act)
        assert rel_err(si.np_f32(a_cache[:, :, rows]), a_u) <= REL_TOL
        assert rel_err(si.np_f32(out[:, rows]), o_u, o_u - o_before) <= REL_TOL


@pytest.mark.parametrize("B,N,D,F,c,k,act", [
    (1, 1024, 256, 1024, 128, 256, 1),     # Tiny (config 0)
    (2, 500, 256, 320, 192, 100, 0),       # ragged chunk, ragged counts
    (1, 192, 128, 128, 192, 1, 1),
])
def test_mlp_overlapped_writeback_matches_plain(cm, oracle, B, N, D, F, c, k, act):
    """App. B.3.3: the activation-cache write-back inside the second GEMM's launch.  Bit for bit the caches of the
    plain entry point, over two chained steps, and within tolerance of the oracle."""
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 6, DEV)
    a_ld = -(-N // 8) * 8 + 8
    NB = -(-N // c)
    o0 = torch.empty_like(x1)
    a0 = torch.zeros((B, F, a_ld), dtype=torch.bfloat16, device=DEV)
    cm.mlp_dense(x1, w1, b1, w2, b2, o0, a0, c, act)
    plain = (a0.clone(), o0.clone())
    over = (a0.clone(), o0.clone())
    a_ref = si.np_f32(a0).astype(np.float64)
    o_ref = si.np_f32(o0).astype(np.float64)
    ws = _u8(cm.mlp_workspace_bytes(B, N, D, F, c, k))
    ws2 = _u8(cm.mlp_overlapped_workspace_bytes(B, N, D, F, c, k))
    assert ws2.numel() == 2 * ws.numel()
    for step in range(2):
        idx, counts = recipes.mlp_indices(B * NB, F, k, 20 + step, DEV, ragged=True)
        idx, counts = idx.view(B, NB, k).contiguous(), counts.view(B, NB).contiguous()
        cm.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, plain[0], plain[1], c, act, ws)
        cm.mlp_sparse_delta_overlapped(x2, w1, b1, w2, idx, counts, over[0], over[1], c, act, ws2)
        assert torch.equal(over[0], plain[0]) and torch.equal(over[1], plain[1]), step
        o_before = o_ref.copy()
        oracle.mlp_sparse_delta(si.np_f32(x2), si.np_f32(w1), si.np_f32(b1), si.np_f32(w2), idx.cpu().numpy(),
                                counts.cpu().numpy(), a_ref, o_ref, c, act)
        assert rel_err(si.np_f32(over[0])[..., :N], a_ref[..., :N]) <= REL_TOL
        assert rel_err(si.np_f32(over[1]), o_ref, o_ref - o_before) <= REL_TOL
        assert torch.all(over[0][..., N:] == 0)                      # padding of the cache rows untouched
        x2 = si.randn_bf16(tuple(x2.shape), si.generator(90 + step, DEV))


def test_mlp_overlapped_writeback_hunyuan_shape(cm):
    """The launch bench.py times: the same caches as the plain entry point at the full HunyuanVideo shape."""
    cfg = si.CONFIGS["hunyuan"]
    B, D, F, c = cfg["B"], cfg["D"], cfg["F"], cfg["c"]
    N = si.config_tokens(cfg)
    k = si.kept(F, cfg["mlp_keep"])
    NB = -(-N // c)
    x1, x2, w1, b1, w2, b2 = recipes.mlp_inputs(B, N, D, F, 7, DEV)
    o0 = torch.empty_like(x1)
    a0 = torch.zeros((B, F, N), dtype=torch.bfloat16, device=DEV)
    cm.mlp_dense(x1, w1, b1, w2, b2, o0, a0, c, 1)
    idx, counts = recipes.mlp_indices(B * NB, F, k, 7, DEV)
    idx, counts = idx.view(B, NB, k).contiguous(), counts.view(B, NB).contiguous()
    a1, o1 = a0.clone(), o0.clone()
    cm.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, a0, o0, c, 1, _u8(cm.mlp_workspace_bytes(B, N, D, F, c, k)))
    cm.mlp_sparse_delta_overlapped(x2, w1, b1, w2, idx, counts, a1, o1, c, 1,
                                   _u8(cm.mlp_overlapped_workspace_bytes(B, N, D, F, c, k)))
    assert torch.equal(a1, a0) and torch.equal(o1, o0)
