"""The error metric and the input recipes of the GPU parity tests (no test cases here).

One metric, used by every floating-point parity assert:

    rel_err(got, ref, update_ref) = max_i |got_i - ref_i| / max(|ref_i|, rms(ref), rms(update_ref))

Elements smaller than the tensor's RMS are judged on absolute error relative to the RMS.  When the compared tensor is
a merge `out = base + update` (attention: cache + o_scale * delta; MLP: M_cache += delta W2), `update_ref` is the
oracle's own update `ref - base`, and its RMS joins the floor: the kernel computes the update, and where cache and
update nearly cancel the rounding of the update (bf16 probabilities, bf16 deltas) is an error on the update's scale,
not on the scale of the much smaller sum.  Where the update is smaller than the output the floor is rms(ref) as
before.  The recipes below keep the update at least comparable with the output, so that a wrong update cannot hide
under the floor; tests/test_parity_recipes_discriminate.py proves that on the CPU for every recipe: an update that
is 10 % short fails the tolerance.
"""
import math

import numpy as np
import torch

import synth_inputs as si

# Spec tolerance for floating-point outputs (bf16 in, fp32 accumulate).
REL_TOL = 2e-2
# Token-merged pre-activations carry ~16 bits of the chunk mean (split-precision bf16 operands).
SCORE_TOL = 1e-3


def _rms(a):
    a = np.asarray(a, np.float64)
    return float(np.sqrt(np.mean(a * a))) if a.size else 0.0


def rel_err(got, ref, update_ref=None):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    floor = _rms(ref)
    if update_ref is not None:
        floor = max(floor, _rms(update_ref))
    if floor == 0.0:
        return float(np.max(np.abs(got - ref))) if got.size else 0.0
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), floor)))


def short_update(base, ref, fraction=0.9):
    """The mutant every merge test must reject: the base plus only `fraction` of the oracle's update."""
    base = np.asarray(base, np.float64)
    return base + fraction * (np.asarray(ref, np.float64) - base)


# ---- input recipes (seeded; the same functions serve the GPU tests on "cuda" and the CPU proof on "cpu") ----------

def attn_inputs(B, H, N, E, seed, device):
    """q, k, v of the second diffusion step of the synthetic recipe: bf16 [B,H,N,E]."""
    (_, _, _), (q, k, v), _ = si.attn_steps(B, H, N, E, seed, device)
    return q, k, v


def attn_base(shape, k_kept, mode, seed, device):
    """The cache the delta is merged into.  mode "unit": N(0,1) entries (the scale of a dense output's cache under
    cancellation); "zero": out is the delta itself; "delta": N(0,1) * sqrt(e / k_kept), the RMS of a subset-softmax
    delta over k_kept columns with N(0,1) scores and values, so cache and delta weigh the same."""
    if mode == "zero":
        return torch.zeros(shape, dtype=torch.bfloat16, device=device)
    scale = 1.0 if mode == "unit" else math.sqrt(math.e / max(k_kept, 1))
    return si.randn_bf16(shape, si.generator(seed + 9, device), scale)


def attn_indices(units, N, k, seed, device, ragged=False, order="ascending"):
    """idx [units, k] int32, counts [units].  order "ascending": k distinct columns, sorted; "shuffled": the same
    in random order; "duplicates": the first third of each list is repeated over the last third (a multiset)."""
    idx, counts = si.uniform_indices(units, N, k, seed, device)
    if order in ("shuffled", "duplicates"):
        g = si.generator(seed + 31, device)
        shuffle = torch.rand((units, k), generator=g, device=device).argsort(dim=1, stable=True)
        idx = torch.gather(idx, 1, shuffle)
    if order == "duplicates" and k >= 3:
        idx[:, k - k // 3:] = idx[:, :k // 3]
    if ragged:
        counts[0] = 0
        counts[1 % units] = 1
        counts[-1] = max(1, k - 5)
        if units > 3:
            counts[2] = min(k, 33)
            counts[3] = min(k, 64)
    return idx.contiguous(), counts


def mlp_inputs(B, N, D, F, seed, device):
    """x1, x2 (independent draws: the activations change completely between the steps), w1, b1, w2, b2."""
    w1, b1, w2, b2 = si.mlp_weights(D, F, seed, device)
    x1, x2 = si.mlp_steps(B, N, D, seed, device, independent=True)
    return x1, x2, w1, b1, w2, b2


def mlp_indices(units, F, k, seed, device, ragged=False):
    idx, counts = si.uniform_indices(units, F, k, seed, device)
    if ragged and k > 70:
        counts[0] = 0
        counts[-1] = 65
        if units > 1:
            counts[1] = k - 3
    return idx.contiguous(), counts


def attn_block_lists(units, N, n_blocks, seed, device, ragged=False, block=128):
    """blocks [units, n_blocks] int32: distinct 128-column key blocks per unit drawn uniformly, ascending;
    block_counts [units].  With `ragged`: one empty list, one single block, one that ends with the sequence's last
    (possibly partial) block, one that lists a block twice."""
    total = -(-N // block)
    g = si.generator(seed + 6000003, device)
    keys = torch.rand((units, total), generator=g, device=device)
    blocks = keys.argsort(dim=1, stable=True)[:, :n_blocks].sort(dim=1).values.to(torch.int32).contiguous()
    counts = torch.full((units,), n_blocks, dtype=torch.int32, device=device)
    if ragged:
        counts[0] = 0
        counts[1 % units] = 1
        blocks[-1, n_blocks - 1] = total - 1            # the last block of the sequence (cut at N)
        if units > 2 and n_blocks > 1:
            blocks[2, 1] = blocks[2, 0]                 # a repeated block counts twice
    return blocks, counts


def expand_block_lists(blocks, counts, N, block=128):
    """The column lists Alg. 3 would be handed for these block lists: every column of every listed block, in list
    order, cut at N.  Returns idx [units, k_stride] int32 (numpy), counts [units]."""
    blocks = np.asarray(blocks)
    counts = np.asarray(counts)
    units, stride = blocks.shape
    idx = np.zeros((units, max(stride * block, 1)), np.int32)
    out_counts = np.zeros(units, np.int32)
    for u in range(units):
        cols = [c for b in blocks[u, :counts[u]] for c in range(int(b) * block, min(N, (int(b) + 1) * block))]
        idx[u, :len(cols)] = cols
        out_counts[u] = len(cols)
    return idx, out_counts
