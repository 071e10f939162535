"""Pins for the oracle's attention and MLP routines.  CPU only.

Attention: Sec. 3.3.1 (dense step, column sums D, O_cache, sparse delta step), Alg. 2-3.
MLP: Sec. 3.3.2, App. B.3.1, Alg. 5-7, and Eq. 2 (subtract-then-add form).

The oracle is compared with library routines (torch scaled_dot_product_attention,
torch GELU and matmul in float64), closed forms, and invariants of the
definitions.  Nothing here is a second copy of the oracle's own loops.
"""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si


def _rand(shape, seed, scale=1.0):
    g = si.generator(seed)
    return si.np_f32(si.randn_bf16(shape, g, scale))


def _t64(a):
    return torch.from_numpy(np.asarray(a)).double()


# ------------------------------------------------------------ attention ----

@pytest.mark.parametrize("B,H,N,E,c", [(1, 2, 96, 16, 32), (2, 1, 70, 8, 32)])
def test_dense_attention_is_textbook_sdpa(oracle, B, H, N, E, c):
    q, k, v = (_rand((B, H, N, E), s) for s in (1, 2, 3))
    scale = 1.0 / math.sqrt(E)
    out, D = oracle.attn_dense(q, k, v, c, scale, want_colsum=True)
    ref = torch.nn.functional.scaled_dot_product_attention(_t64(q), _t64(k), _t64(v))  # default scale 1/sqrt(E)
    assert np.allclose(out, ref.numpy(), rtol=0, atol=1e-12)
    # D against the definition  D[i,j] = sum_{q in chunk i} P[q,j]  built from torch.softmax
    P = torch.softmax(_t64(q) @ _t64(k).transpose(-1, -2) * scale, dim=-1).numpy()
    NB = -(-N // c)
    for i in range(NB):
        assert np.allclose(D[:, :, i], P[:, :, i * c:(i + 1) * c].sum(axis=2), rtol=0, atol=1e-12)
    # rows of P sum to one  =>  each row of D sums to the number of query rows in its chunk
    rows = np.array([min(c, N - i * c) for i in range(NB)], np.float64)
    assert np.allclose(D.sum(axis=-1), rows[None, None, :], rtol=0, atol=1e-10)


def test_dense_attention_operand_roles(oracle):
    """A transposed operand or a swapped k/v shows here: keys and queries of different counts."""
    B, H, Nq, Nk, E, c = 1, 1, 40, 56, 8, 16
    q = _rand((B, H, Nq, E), 4)
    k, v = _rand((B, H, Nk, E), 5), _rand((B, H, Nk, E), 6)
    out = oracle.attn_dense(q, k, v, c, 0.3)
    ref = torch.softmax(_t64(q) @ _t64(k).transpose(-1, -2) * 0.3, dim=-1) @ _t64(v)
    assert np.allclose(out, ref.numpy(), rtol=0, atol=1e-12)


def _sparse_setup(seed=7, B=1, H=2, N=80, E=16, c=32, kk=9):
    q, k, v = (_rand((B, H, N, E), seed + s) for s in range(3))
    NB = -(-N // c)
    idx_t, cnt_t = si.uniform_indices(B * H * NB, N, kk, seed)
    idx = idx_t.numpy().reshape(B, H, NB, kk).copy()
    counts = cnt_t.numpy().reshape(B, H, NB).copy()
    base = np.ascontiguousarray(_rand((B, H, N, E), seed + 5).astype(np.float64))
    return q, k, v, idx, counts, base, c, 1.0 / math.sqrt(E)


def test_sparse_delta_all_columns_is_dense(oracle):
    """k = N reproduces dense attention (Sec. 3.3.1, last paragraph)."""
    B, H, N, E, c = 1, 2, 70, 16, 32
    q, k, v = (_rand((B, H, N, E), s) for s in (11, 12, 13))
    NB = -(-N // c)
    rng = np.random.default_rng(0)
    idx = np.stack([rng.permutation(N) for _ in range(B * H * NB)]).astype(np.int32).reshape(B, H, NB, N)
    counts = np.full((B, H, NB), N, np.int32)
    zero = np.zeros((B, H, N, E))
    out = oracle.attn_sparse_delta(q, k, v, idx, counts, zero, c, 1 / math.sqrt(E), 1.0)
    ref = torch.nn.functional.scaled_dot_product_attention(_t64(q), _t64(k), _t64(v)).numpy()
    assert np.allclose(out, ref, rtol=0, atol=1e-12)


def test_sparse_delta_counts_zero_and_single_column(oracle):
    q, k, v, idx, counts, base, c, scale = _sparse_setup()
    counts0 = np.zeros_like(counts)
    out = oracle.attn_sparse_delta(q, k, v, idx, counts0, base, c, scale, 1.0)
    assert np.array_equal(out, base)                               # nothing selected: the cache, bit for bit
    # one selected column: softmax over one entry is 1, so delta = V_j exactly
    counts1 = np.ones_like(counts)
    out = oracle.attn_sparse_delta(q, k, v, idx, counts1, np.zeros_like(base), c, scale, 1.0)
    B, H, N, E = q.shape
    for b in range(B):
        for h in range(H):
            for i in range(idx.shape[2]):
                j = idx[b, h, i, 0]
                blk = out[b, h, i * c:(i + 1) * c]
                assert np.array_equal(blk, np.broadcast_to(v[b, h, j].astype(np.float64), blk.shape))


def test_sparse_delta_subset_softmax_identity_and_scale(oracle):
    """p^S_j = P_qj / sum_{j' in S} P_qj'  links the subset softmax to the dense one; o_scale is linear."""
    q, k, v, idx, counts, base, c, scale = _sparse_setup(seed=21, kk=13)
    counts[0, 1, 1] = 5                                            # ragged counts
    B, H, N, E = q.shape
    P = torch.softmax(_t64(q) @ _t64(k).transpose(-1, -2) * scale, dim=-1).numpy()
    ref = np.empty_like(base)
    for b in range(B):
        for h in range(H):
            for i in range(idx.shape[2]):
                S = idx[b, h, i, :counts[b, h, i]]
                rows = slice(i * c, min(N, (i + 1) * c))
                w = P[b, h, rows][:, S]
                w = w / w.sum(axis=1, keepdims=True)
                ref[b, h, rows] = w @ v[b, h, S].astype(np.float64)
    for o_scale in (1.0, -1.0, 0.5):
        out = oracle.attn_sparse_delta(q, k, v, idx, counts, base, c, scale, o_scale)
        assert np.allclose(out, base + o_scale * ref, rtol=0, atol=1e-11)
    # all-ones V: probabilities over S sum to one
    ones = np.ones_like(v)
    out = oracle.attn_sparse_delta(q, k, ones, idx, counts, np.zeros_like(base), c, scale, 1.0)
    assert np.allclose(out, 1.0, rtol=0, atol=1e-13)
    # the scale matters (a dropped 1/sqrt(E) shows here)
    out2 = oracle.attn_sparse_delta(q, k, v, idx, counts, base, c, 2 * scale, 1.0)
    assert not np.allclose(out2, base + ref, atol=1e-3)


def test_sparse_delta_order_of_S_and_cache_roundtrip(oracle):
    q, k, v, idx, counts, base, c, scale = _sparse_setup(seed=31, kk=11)
    out = oracle.attn_sparse_delta(q, k, v, idx, counts, base, c, scale, 1.0)
    idx_rev = np.ascontiguousarray(idx[..., ::-1])
    out_rev = oracle.attn_sparse_delta(q, k, v, idx_rev, counts, base, c, scale, 1.0)
    assert np.allclose(out, out_rev, rtol=0, atol=1e-13)           # S is a set
    # dense step builds O_cache = O_dense - Delta (o_scale = -1); a sparse step with the same q,k,v gives O_dense back
    dense = oracle.attn_dense(q, k, v, c, scale)
    o_cache = oracle.attn_sparse_delta(q, k, v, idx, counts, dense, c, scale, -1.0)
    again = oracle.attn_sparse_delta(q, k, v, idx, counts, o_cache, c, scale, 1.0)
    assert np.allclose(again, dense, rtol=0, atol=1e-13)
    assert not np.allclose(o_cache, dense, atol=1e-3)
    # each chunk uses its own index row: swapping two chunks' rows changes those chunks only
    idx_sw = idx.copy()
    idx_sw[0, 0, 0], idx_sw[0, 0, 1] = idx[0, 0, 1], idx[0, 0, 0]
    out_sw = oracle.attn_sparse_delta(q, k, v, idx_sw, counts, base, c, scale, 1.0)
    assert np.array_equal(out_sw[0, 0, 2 * c:], out[0, 0, 2 * c:]) and np.array_equal(out_sw[0, 1], out[0, 1])
    assert not np.allclose(out_sw[0, 0, :2 * c], out[0, 0, :2 * c], atol=1e-6)


def test_row_stats_and_stale_column_sums(oracle):
    """Alg. 4: p_approx = exp(qk - prev_m) / prev_l summed over each chunk's rows.
    Pins: the statistics against torch.logsumexp (m + log l is the row's log-sum-exp, whatever reference m is used);
    with the current step's own statistics the sums are the exact column sums D of the dense step (softmax from
    torch); any other valid reference pair (m - d, l e^d) gives the same sums; doubling prev_l halves them; and
    with step-1 statistics on step-2 inputs the sums equal torch's exp/sum written from the definition."""
    B, H, N, E, c = 2, 2, 70, 16, 32
    q, k = _rand((B, H, N, E), 21), _rand((B, H, N, E), 22)
    scale = 1.0 / math.sqrt(E)
    m, l = oracle.attn_row_stats(q, k, scale)
    S = _t64(q) @ _t64(k).transpose(-1, -2) * scale
    assert np.allclose(m, S.max(dim=-1).values.numpy(), rtol=0, atol=1e-12)
    assert np.allclose(m + np.log(l), torch.logsumexp(S, dim=-1).numpy(), rtol=0, atol=1e-12)
    NB = -(-N // c)
    P = torch.softmax(S, dim=-1).numpy()
    D_def = np.stack([P[:, :, i * c:(i + 1) * c].sum(axis=2) for i in range(NB)], axis=2)
    cs = oracle.attn_colsum_stale(q, k, m, l, c, scale)
    assert cs.shape == (B, H, NB, N)
    assert np.allclose(cs, D_def, rtol=0, atol=1e-12)
    _, D = oracle.attn_dense(q, k, _rand((B, H, N, E), 23), c, scale, want_colsum=True)
    assert np.allclose(cs, D, rtol=0, atol=1e-12)
    assert np.allclose(oracle.attn_colsum_stale(q, k, m - 1.5, l * math.exp(1.5), c, scale), cs, rtol=1e-12, atol=0)
    assert np.allclose(oracle.attn_colsum_stale(q, k, m, 2.0 * l, c, scale), 0.5 * cs, rtol=1e-12, atol=0)
    # stale statistics: step-2 inputs with the step-1 normalisers
    q2 = q + _rand((B, H, N, E), 24, 0.05)
    k2 = k + _rand((B, H, N, E), 25, 0.05)
    S2 = _t64(q2) @ _t64(k2).transpose(-1, -2) * scale
    approx = (torch.exp(S2 - _t64(m).unsqueeze(-1)) / _t64(l).unsqueeze(-1)).numpy()
    ref = np.stack([approx[:, :, i * c:(i + 1) * c].sum(axis=2) for i in range(NB)], axis=2)
    got = oracle.attn_colsum_stale(q2, k2, m, l, c, scale)
    assert np.allclose(got, ref, rtol=1e-12, atol=0)
    assert not np.allclose(got, cs, rtol=1e-3, atol=0)   # the stale sums are an approximation, not D itself
    # a transposed operand (k, q swapped) must show: rows and columns are different axes
    assert not np.allclose(oracle.attn_colsum_stale(k, q, m, l, c, scale), cs, rtol=1e-3, atol=0)


def test_sparse_delta_rejects_bad_indices(oracle):
    q, k, v, idx, counts, base, c, scale = _sparse_setup()
    bad = idx.copy()
    bad[0, 0, 0, 0] = q.shape[2]
    with pytest.raises(ValueError):
        oracle.attn_sparse_delta(q, k, v, bad, counts, base, c, scale, 1.0)


# ------------------------------------------------------------------ MLP ----

def _gelu(x, act):
    return torch.nn.functional.gelu(x, approximate="none" if act == 0 else "tanh")


def _mlp_setup(seed=3, B=2, N=50, D=16, F=40, c=16):
    x = _rand((B, N, D), seed)
    w1 = _rand((F, D), seed + 1, 1 / math.sqrt(D))
    b1 = _rand((F,), seed + 2, 0.1)
    w2 = _rand((F, D), seed + 3, 1 / math.sqrt(F))
    b2 = _rand((D,), seed + 4, 0.1)
    return x, w1, b1, w2, b2, c


@pytest.mark.parametrize("act", [0, 1])
def test_dense_mlp_is_textbook(oracle, act):
    x, w1, b1, w2, b2, c = _mlp_setup()
    out, a_cache, T_m = oracle.mlp_dense(x, w1, b1, w2, b2, c, act, a_ld=x.shape[1] + 3)
    pre = _t64(x) @ _t64(w1).T
    A = _gelu(pre + _t64(b1), act)
    ref = A @ _t64(w2) + _t64(b2)
    assert np.allclose(out, ref.numpy(), rtol=0, atol=1e-12)
    N = x.shape[1]
    assert np.allclose(a_cache[:, :, :N], A.transpose(1, 2).numpy(), rtol=0, atol=1e-12)   # neuron-major cache
    assert np.all(a_cache[:, :, N:] == 0)
    NB = -(-N // c)
    for i in range(NB):                                            # T_m: chunk mean of the pre-activation, no bias
        assert np.allclose(T_m[:, i], pre[:, i * c:(i + 1) * c].mean(dim=1).numpy(), rtol=0, atol=1e-12)
    # no biases
    out0 = oracle.mlp_dense(x, w1, None, w2, None, c, act, want_caches=False)
    assert np.allclose(out0, (_gelu(pre, act) @ _t64(w2)).numpy(), rtol=0, atol=1e-12)


def test_gelu_variants_differ_and_known_values(oracle):
    """One token, one neuron, D = 1: out = gelu(x w1 + b1) w2 + b2 in closed form."""
    x = np.array([[[1.0]]], np.float32)
    w1 = np.array([[2.0]], np.float32)
    b1 = np.array([-1.0], np.float32)
    w2 = np.array([[3.0]], np.float32)
    b2 = np.array([0.5], np.float32)
    e = oracle.mlp_dense(x, w1, b1, w2, b2, 1, 0, want_caches=False)[0, 0, 0]
    t = oracle.mlp_dense(x, w1, b1, w2, b2, 1, 1, want_caches=False)[0, 0, 0]
    assert abs(e - (0.5 * (1 + math.erf(1 / math.sqrt(2))) * 3 + 0.5)) < 1e-15      # gelu(1) = Phi(1)
    g_tanh = 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * (1 + 0.044715)))
    assert abs(t - (g_tanh * 3 + 0.5)) < 1e-15
    assert abs(e - t) > 1e-5


def test_tile_scores_linearity(oracle):
    """mean_c(X) @ W1^T = mean_c(X @ W1^T): Alg. 7's score equals Alg. 5's cached tile mean when X is unchanged."""
    x, w1, b1, w2, b2, c = _mlp_setup(seed=9)
    T = oracle.mlp_tile_scores(x, w1, c)
    _, _, T_m = oracle.mlp_dense(x, w1, b1, w2, b2, c, 0)
    assert np.allclose(T, T_m, rtol=0, atol=1e-12)
    N = x.shape[1]
    NB = -(-N // c)
    xm = np.stack([x[:, i * c:(i + 1) * c].astype(np.float64).mean(axis=1) for i in range(NB)], axis=1)
    assert np.allclose(T, xm @ w1.astype(np.float64).T, rtol=0, atol=1e-12)       # last chunk: mean over its real rows


@pytest.mark.parametrize("act", [0, 1])
def test_sparse_mlp_all_columns_is_dense(oracle, act):
    x1, w1, b1, w2, b2, c = _mlp_setup(seed=13)
    x2 = _rand(x1.shape, 99)
    B, N, D = x1.shape
    F = w1.shape[0]
    o_cache, a_cache, _ = oracle.mlp_dense(x1, w1, b1, w2, b2, c, act)
    NB = -(-N // c)
    rng = np.random.default_rng(0)
    idx = np.stack([rng.permutation(F) for _ in range(B * NB)]).astype(np.int32).reshape(B, NB, F)
    counts = np.full((B, NB), F, np.int32)
    oracle.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, a_cache, o_cache, c, act)
    A2 = _gelu(_t64(x2) @ _t64(w1).T + _t64(b1), act)
    ref = A2 @ _t64(w2) + _t64(b2)
    assert np.allclose(o_cache, ref.numpy(), rtol=0, atol=1e-11)
    assert np.allclose(a_cache, A2.transpose(1, 2).numpy(), rtol=0, atol=1e-12)


def test_sparse_mlp_is_equation_2_and_keeps_cache_invariant(oracle):
    """One pass (App. B.3.1) equals subtract-then-add (Eq. 2), and after any sequence of sparse
    steps  O_cache = A_cache^T W2 + b2  still holds."""
    act = 1
    x1, w1, b1, w2, b2, c = _mlp_setup(seed=17, B=2, N=45, D=12, F=30, c=16)
    B, N, D = x1.shape
    F = w1.shape[0]
    NB = -(-N // c)
    o_cache, a_cache, _ = oracle.mlp_dense(x1, w1, b1, w2, b2, c, act)
    o1 = o_cache.copy()
    xs = [_rand(x1.shape, 200 + s) for s in range(3)]
    kk = 7
    A_prev = _gelu(_t64(x1) @ _t64(w1).T + _t64(b1), act).numpy()                 # [B,N,F]
    o_expect = o1.copy()
    for step, x2 in enumerate(xs):
        idx_t, cnt_t = si.uniform_indices(B * NB, F, kk, 50 + step)
        idx = idx_t.numpy().reshape(B, NB, kk).copy()
        counts = cnt_t.numpy().reshape(B, NB).copy()
        counts[0, 0] = 0
        counts[1, NB - 1] = 3
        A2 = _gelu(_t64(x2) @ _t64(w1).T + _t64(b1), act).numpy()
        M = np.zeros((B, N, F))
        for b in range(B):
            for i in range(NB):
                M[b, i * c:(i + 1) * c, idx[b, i, :counts[b, i]]] = 1.0
        # Eq. 2: o2 = o1 - (A_prev * M) W2 + (A2 * M) W2
        o_expect = o_expect - (A_prev * M) @ w2.astype(np.float64) + (A2 * M) @ w2.astype(np.float64)
        A_prev = np.where(M > 0, A2, A_prev)
        oracle.mlp_sparse_delta(x2, w1, b1, w2, idx, counts, a_cache, o_cache, c, act)
        assert np.allclose(o_cache, o_expect, rtol=0, atol=1e-11)
        assert np.allclose(a_cache, A_prev.transpose(0, 2, 1), rtol=0, atol=1e-12)
        inv = np.einsum("bfn,fd->bnd", a_cache, w2.astype(np.float64)) + b2.astype(np.float64)
        assert np.allclose(o_cache, inv, rtol=0, atol=1e-11)


def test_sparse_mlp_noop_cases(oracle):
    act = 0
    x1, w1, b1, w2, b2, c = _mlp_setup(seed=23)
    B, N, D = x1.shape
    F = w1.shape[0]
    NB = -(-N // c)
    o_cache, a_cache, _ = oracle.mlp_dense(x1, w1, b1, w2, b2, c, act)
    o0, a0 = o_cache.copy(), a_cache.copy()
    idx_t, cnt_t = si.uniform_indices(B * NB, F, 9, 5)
    idx = idx_t.numpy().reshape(B, NB, 9).copy()
    counts = cnt_t.numpy().reshape(B, NB).copy()
    # counts = 0: both caches untouched, bit for bit
    oracle.mlp_sparse_delta(_rand(x1.shape, 77), w1, b1, w2, idx, np.zeros_like(counts), a_cache, o_cache, c, act)
    assert np.array_equal(o_cache, o0) and np.array_equal(a_cache, a0)
    # x unchanged since the dense step: delta = 0 for any S
    oracle.mlp_sparse_delta(x1, w1, b1, w2, idx, counts, a_cache, o_cache, c, act)
    assert np.allclose(o_cache, o0, rtol=0, atol=1e-13) and np.allclose(a_cache, a0, rtol=0, atol=1e-14)
    # without b1 the activations differ (the bias is inside the activation)
    o_nb, a_nb = o0.copy(), a0.copy()
    oracle.mlp_sparse_delta(x1, w1, None, w2, idx, counts, a_nb, o_nb, c, act)
    assert not np.allclose(o_nb, o0, atol=1e-4)
