"""Pins for the oracle's voxel reorder (Alg. 1) and top-k column selection
(Sec. 3.3.1 TopK_k(D); Alg. 7 TopK(|T - T_m|)).  CPU only.

Each check compares the oracle with something other than itself: hand-worked
permutations, numpy's reshape/transpose, bijection and round-trip properties,
brute-force selection, numpy's argmax/argsort, and symmetry arguments.
"""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _golden_perms():
    cases = []
    with open(os.path.join(GOLD, "voxel_perm_examples.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            left, right = line.split(":")
            cases.append((tuple(int(t) for t in left.split()), [int(t) for t in right.split()]))
    return cases


@pytest.mark.parametrize("args,expected", _golden_perms())
def test_voxel_perm_worked_examples(oracle, args, expected):
    perm, inv = oracle.voxel_perm(*args)
    assert perm.tolist() == expected
    assert inv[perm].tolist() == list(range(len(expected)))


@pytest.mark.parametrize("T,H,W,vt,vh,vw", [(8, 8, 16, 4, 4, 8), (4, 6, 8, 2, 3, 4), (1, 64, 64, 1, 8, 8), (6, 4, 10, 3, 2, 5)])
def test_voxel_perm_divisible_equals_rearrange(oracle, T, H, W, vt, vh, vw):
    """Alg. 1's rearrange pattern written with numpy reshape/transpose."""
    perm, inv = oracle.voxel_perm(0, T, H, W, 0, vt, vh, vw)
    ids = np.arange(T * H * W).reshape(T // vt, vt, H // vh, vh, W // vw, vw)
    expect = ids.transpose(0, 2, 4, 1, 3, 5).reshape(-1)
    assert np.array_equal(perm, expect)
    # data version, with a batch and a feature axis
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, T * H * W, 3)).astype(np.float32)
    xr = x.reshape(2, T // vt, vt, H // vh, vh, W // vw, vw, 3).transpose(0, 1, 3, 5, 2, 4, 6, 7).reshape(2, -1, 3)
    y = oracle.reorder_rows(x, perm, inverse=False)
    assert np.array_equal(y, xr)
    assert np.array_equal(oracle.reorder_rows(y, perm, inverse=True), x)
    # reverse_voxel_order = the inverse rearrange
    back = xr.reshape(2, T // vt, H // vh, W // vw, vt, vh, vw, 3).transpose(0, 1, 4, 2, 5, 3, 6, 7).reshape(2, -1, 3)
    assert np.array_equal(back, x)


@pytest.mark.parametrize("npre,T,H,W,nsuf,vt,vh,vw", [
    (0, 30, 48, 80, 256, 4, 6, 8),    # HunyuanVideo-shaped: T=30 does not divide by 4
    (0, 21, 45, 80, 0, 4, 6, 8),      # WAN-shaped: 21 and 45 do not divide
    (512, 1, 64, 64, 0, 1, 8, 8),     # FLUX-shaped: text prefix
    (3, 5, 7, 9, 2, 2, 3, 4),
])
def test_voxel_perm_structure(oracle, npre, T, H, W, nsuf, vt, vh, vw):
    perm, inv = oracle.voxel_perm(npre, T, H, W, nsuf, vt, vh, vw)
    N = npre + T * H * W + nsuf
    assert perm.shape == (N,)
    assert np.array_equal(np.sort(perm), np.arange(N))            # bijection
    assert np.array_equal(inv[perm], np.arange(N))                 # inverse
    assert np.array_equal(perm[inv], np.arange(N))
    assert np.array_equal(perm[:npre], np.arange(npre))            # prefix untouched
    assert np.array_equal(perm[N - nsuf:], np.arange(N - nsuf, N)) # suffix untouched
    vol = vt * vh * vw
    n_full = (T // vt) * (H // vh) * (W // vw)
    grid = perm[npre:npre + T * H * W] - npre
    t, h, w = grid // (H * W), (grid // W) % H, grid % W
    for vidx in range(0, n_full, max(1, n_full // 50)):            # each full voxel = one contiguous run
        sl = slice(vidx * vol, (vidx + 1) * vol)
        assert t[sl].max() - t[sl].min() == vt - 1 and t[sl].min() % vt == 0
        assert h[sl].max() - h[sl].min() == vh - 1 and h[sl].min() % vh == 0
        assert w[sl].max() - w[sl].min() == vw - 1 and w[sl].min() % vw == 0
        assert len(set(zip(t[sl].tolist(), h[sl].tolist(), w[sl].tolist()))) == vol
    rem = grid[n_full * vol:]                                       # remainder: raster order, outside full voxels
    assert np.all(np.diff(rem) > 0)
    tr, hr, wr = rem // (H * W), (rem // W) % H, rem % W
    assert np.all((tr >= (T // vt) * vt) | (hr >= (H // vh) * vh) | (wr >= (W // vw) * vw))
    # voxels come in (tc, hc, wc) lexicographic order
    firsts = grid[0:n_full * vol:vol]
    key = ((firsts // (H * W)) // vt) * (H // vh) * (W // vw) + (((firsts // W) % H) // vh) * (W // vw) + (firsts % W) // vw
    assert np.array_equal(key, np.arange(n_full))


def test_reorder_rows_bytes(oracle):
    perm, inv = oracle.voxel_perm(1, 2, 4, 4, 2, 2, 2, 2)
    N = perm.size
    x = np.arange(2 * N * 5, dtype=np.uint8).reshape(2, N, 5)
    y = oracle.reorder_rows(x, perm)
    assert np.array_equal(y, x[:, perm])                           # dst[new] = src[perm[new]]
    z = oracle.reorder_rows(x, perm, inverse=True)
    assert np.array_equal(z, x[:, inv])                            # numpy fancy indexing as the library routine
    assert np.array_equal(oracle.reorder_rows(y, perm, inverse=True), x)


# ---------------------------------------------------------------- top-k ----

def _brute_topk(score, k):
    """Repeated arg-max selection, lowest column first among equals; O(C k)."""
    s = [float(v) for v in score]
    taken = []
    alive = [True] * len(s)
    for _ in range(k):
        best = -1
        for j in range(len(s)):
            if alive[j] and (best < 0 or s[j] > s[best]):
                best = j
        alive[best] = False
        taken.append(best)
    return sorted(taken)


@pytest.mark.parametrize("with_prev", [False, True])
def test_topk_brute_force_tiny(oracle, with_prev):
    rng = np.random.default_rng(1)
    for C, k in [(7, 3), (16, 16), (33, 1), (40, 11), (5, 0)]:
        cur = rng.standard_normal((6, C)).astype(np.float32)
        prev = rng.standard_normal((6, C)).astype(np.float32) if with_prev else None
        idx, counts = oracle.topk_cols(cur, prev, k, k_stride=k + 2)
        assert counts.tolist() == [k] * 6
        score = np.abs(cur - prev) if with_prev else cur
        for r in range(6):
            assert idx[r, :k].tolist() == _brute_topk(score[r], k)
            assert idx[r, k:].tolist() == [-1, -1]                 # slots beyond k untouched


def test_topk_ties_lower_column_wins(oracle):
    cur = np.array([[1, 3, 3, 2, 3, 0, 3, 1]], np.float32)
    idx, _ = oracle.topk_cols(cur, None, 2)
    assert idx.tolist() == [[1, 2]]
    idx, _ = oracle.topk_cols(cur, None, 3)
    assert idx.tolist() == [[1, 2, 4]]
    idx, _ = oracle.topk_cols(cur, None, 5)
    assert idx.tolist() == [[1, 2, 3, 4, 6]]
    # with prev: |cur - prev| ties, and +0 / -0 equal
    cur = np.array([[0.5, -0.5, 0.0, -0.0, 0.25]], np.float32)
    prev = np.zeros_like(cur)
    idx, _ = oracle.topk_cols(cur, prev, 1)
    assert idx.tolist() == [[0]]
    idx, _ = oracle.topk_cols(cur, prev, 4)
    assert idx.tolist() == [[0, 1, 2, 4]]


def test_topk_special_cases_and_library(oracle):
    rng = np.random.default_rng(2)
    R, C = 5, 301
    cur = rng.permutation(R * C).reshape(R, C).astype(np.float32)  # all distinct
    idx, _ = oracle.topk_cols(cur, None, C)
    assert np.array_equal(idx, np.tile(np.arange(C, dtype=np.int32), (R, 1)))      # k = C keeps everything
    idx, _ = oracle.topk_cols(cur, None, 1)
    assert np.array_equal(idx[:, 0], np.argmax(cur, axis=1))                       # k = 1 is argmax
    for k in (2, 37, 150, 300):
        idx, _ = oracle.topk_cols(cur, None, k)
        lib = np.sort(np.argsort(-cur, axis=1, kind="stable")[:, :k], axis=1)      # numpy sort as the library routine
        assert np.array_equal(idx, lib)
        # a column permutation permutes the answer
        p = rng.permutation(C)
        idx_p, _ = oracle.topk_cols(np.ascontiguousarray(cur[:, p]), None, k)
        for r in range(R):
            assert sorted(p[idx_p[r]].tolist()) == idx[r].tolist()
    prev = rng.standard_normal((R, C)).astype(np.float32)
    idx, _ = oracle.topk_cols(cur, prev, 20)
    lib = np.sort(np.argsort(-np.abs(cur - prev), axis=1, kind="stable")[:, :20], axis=1)
    assert np.array_equal(idx, lib)
    # the sign of the difference does not matter, the order of subtraction neither
    idx2, _ = oracle.topk_cols(prev, cur, 20)
    assert np.array_equal(idx, idx2)


def test_topk_float_decision(oracle):
    """The score |cur - prev| is one float32 subtract: differences that vanish in
    float32 tie (and the lower column wins) although they differ in float64."""
    cur = np.array([[1.0 + 2.0 ** -23, 1.0, 1.0]], np.float32)
    prev = np.array([[2.0 ** -30, 0.0, -(2.0 ** -25)]], np.float32)
    # float32: col0 = fl(1 + 2^-23 - 2^-30) = 1 + 2^-23; col1 = 1; col2 = fl(1 + 2^-25) = 1.
    # In float64 col2 would beat col1; in float32 they tie and the lower column wins.
    assert np.abs(cur.astype(np.float64) - prev.astype(np.float64))[0, 2] > 1.0
    idx, _ = oracle.topk_cols(cur, prev, 2)
    assert idx.tolist() == [[0, 1]]


def test_topk_rejects_bad_arguments(oracle):
    cur = np.zeros((2, 4), np.float32)
    with pytest.raises(ValueError):
        oracle.topk_cols(cur, None, 5)
    with pytest.raises(ValueError):
        oracle.topk_cols(cur, None, 3, k_stride=2)


# ----------------------------------------------------------------- bit-packed masks ---

@pytest.mark.parametrize("R,C", [(3, 1), (4, 31), (4, 32), (5, 33), (3, 1000), (2, 4608)])
def test_mask_conversions_against_numpy(oracle, R, C):
    """App. B.4 / Table 3: a bit-packed row and its index list, against numpy's packbits / nonzero."""
    rng = np.random.default_rng(C)
    dense = rng.random((R, C)) < 0.3
    dense[0] = False                                        # an empty row
    dense[-1] = True                                        # a full row
    words = -(-C // 32)
    padded = np.zeros((R, words * 32), bool)
    padded[:, :C] = dense
    packed = np.packbits(padded, axis=1, bitorder="little").view(np.uint32).reshape(R, words)
    k_stride = C
    idx, counts = oracle.mask_to_indices(np.ascontiguousarray(packed), C, k_stride)
    for r in range(R):
        want = np.nonzero(dense[r])[0]
        assert counts[r] == len(want) and np.array_equal(idx[r, :counts[r]], want)
        assert (idx[r, counts[r]:] == -1).all()             # the rest of the row is untouched
    # the inverse, with rubbish in the padding bits of the destination and out-of-range / repeated entries in the list
    idx2 = np.concatenate([idx, np.full((R, 3), -1, np.int32)], axis=1)
    idx2[:, -3] = np.where(counts > 0, idx[:, 0], -5)       # a repeat of the first entry (or a negative column)
    idx2[:, -2] = C + 7                                     # beyond the last column
    idx2 = np.ascontiguousarray(np.roll(idx2, 3, axis=1))   # rubbish first: the list is unsorted now
    back = oracle.indices_to_mask(idx2, (counts + 3).astype(np.int32), C, fill=0xffffffff)
    assert np.array_equal(back, packed)
    # a list shorter than the mask's population keeps the first k_stride columns
    short, short_counts = oracle.mask_to_indices(np.ascontiguousarray(packed), C, max(1, C // 8))
    for r in range(R):
        want = np.nonzero(dense[r])[0][:max(1, C // 8)]
        assert short_counts[r] == len(want) and np.array_equal(short[r, :short_counts[r]], want)


def test_mask_ignores_bits_beyond_the_last_column(oracle):
    packed = np.full((2, 2), 0xffffffff, np.uint32)
    idx, counts = oracle.mask_to_indices(packed, 40, 64)
    assert counts.tolist() == [40, 40] and np.array_equal(idx[0, :40], np.arange(40))
