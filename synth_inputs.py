"""Seeded synthetic inputs shared by the oracle tests, the GPU parity tests and bench.py.

This module holds no arithmetic of the method itself: only shapes, random
draws and the bf16 storage format.  Real model activations (FLUX.1-dev,
HunyuanVideo, WAN2.1) need weights that are not available here; tensors with
those models' shapes and the cross-step change structure below stand in.

Recipe (all draws from one torch.Generator seeded with `seed`):
  step-1 tensors  q1,k1,v1,x1 ~ N(0,1); w1 ~ N(0,1)/sqrt(D); w2 ~ N(0,1)/sqrt(F);
                  b1,b2 ~ 0.1 N(0,1); everything rounded to bf16.
  step-2 tensors  a random 15 % of the columns (key tokens for attention,
                  hidden neurons for the MLP score source) are "hot":
                  k2,v2 = k1,v1 + 0.1 N(0,1) on hot rows, + 0.01 N(0,1) elsewhere;
                  q2 = q1 + 0.01 N(0,1); x2 = x1 + 0.01 N(0,1).
  MLP top-k score source: cur = prev + 0.1 N(0,1) on hot neurons and
                  + 0.01 N(0,1) elsewhere (float32).
"""
import math

import numpy as np
import torch

HOT_FRACTION = 0.15
HOT_SIGMA = 0.1
COLD_SIGMA = 0.01

# name -> shapes of the benchmark configurations (0 Tiny, 1 FLUX, 2 HunyuanVideo, 3 WAN2.1-14B)
CONFIGS = {
    "tiny": dict(B=1, H=2, E=64, c=128, n_prefix=0, grid=(8, 8, 16), n_suffix=0, voxel=(4, 4, 8),
                 D=256, F=1024, attn_keep=0.25, mlp_keep=0.25),
    "flux": dict(B=1, H=24, E=128, c=192, n_prefix=512, grid=(1, 64, 64), n_suffix=0, voxel=(1, 8, 8),
                 D=3072, F=12288, attn_keep=0.07, mlp_keep=0.10),
    "hunyuan": dict(B=1, H=24, E=128, c=192, n_prefix=0, grid=(30, 48, 80), n_suffix=256, voxel=(4, 6, 8),
                    D=3072, F=12288, attn_keep=0.07, mlp_keep=0.07),
    "wan": dict(B=1, H=40, E=128, c=192, n_prefix=0, grid=(21, 45, 80), n_suffix=0, voxel=(4, 6, 8),
                D=5120, F=13824, attn_keep=0.07, mlp_keep=0.07),
}


def config_tokens(cfg):
    t, h, w = cfg["grid"]
    return cfg["n_prefix"] + t * h * w + cfg["n_suffix"]


def kept(C, keep_fraction):
    """Number of columns kept out of C at a keep fraction (sparsity = 1 - keep)."""
    return max(0, min(C, int(round(keep_fraction * C))))


def generator(seed, device="cpu"):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def randn_bf16(shape, g, scale=1.0):
    x = torch.randn(shape, generator=g, device=g.device, dtype=torch.float32)
    if scale != 1.0:
        x = x * scale
    return x.to(torch.bfloat16)


def hot_mask(C, g):
    """Boolean [C]: a random HOT_FRACTION of the columns."""
    n_hot = int(round(HOT_FRACTION * C))
    order = torch.randperm(C, generator=g, device=g.device)
    m = torch.zeros(C, dtype=torch.bool, device=g.device)
    m[order[:n_hot]] = True
    return m


def perturb_rows(t, hot, g):
    """t [..., C, E] bf16 -> t + sigma N(0,1) with sigma chosen per row of the C axis."""
    sigma = torch.where(hot, HOT_SIGMA, COLD_SIGMA).to(torch.float32).view(*([1] * (t.dim() - 2)), -1, 1)
    noise = torch.randn(t.shape, generator=g, device=g.device, dtype=torch.float32)
    return (t.float() + sigma * noise).to(torch.bfloat16)


def perturb_all(t, g, sigma=COLD_SIGMA):
    noise = torch.randn(t.shape, generator=g, device=g.device, dtype=torch.float32)
    return (t.float() + sigma * noise).to(torch.bfloat16)


def attn_steps(B, H, N, E, seed, device="cpu"):
    """(q1,k1,v1), (q2,k2,v2), hot: bf16 tensors [B,H,N,E] for two consecutive diffusion steps."""
    g = generator(seed, device)
    q1 = randn_bf16((B, H, N, E), g)
    k1 = randn_bf16((B, H, N, E), g)
    v1 = randn_bf16((B, H, N, E), g)
    hot = hot_mask(N, g)
    k2 = perturb_rows(k1, hot, g)
    v2 = perturb_rows(v1, hot, g)
    q2 = perturb_all(q1, g)
    return (q1, k1, v1), (q2, k2, v2), hot


def mlp_weights(D, F, seed, device="cpu"):
    """w1 [F,D], b1 [F], w2 [F,D], b2 [D] in bf16."""
    g = generator(seed + 1000003, device)
    w1 = randn_bf16((F, D), g, 1.0 / math.sqrt(D))
    b1 = randn_bf16((F,), g, 0.1)
    w2 = randn_bf16((F, D), g, 1.0 / math.sqrt(F))
    b2 = randn_bf16((D,), g, 0.1)
    return w1, b1, w2, b2


def mlp_steps(B, N, D, seed, device="cpu", independent=False):
    """x1, x2: bf16 [B,N,D] for two consecutive diffusion steps.  With `independent` the second step is a fresh
    N(0,1) draw instead of a small perturbation of the first: the change of the activations is then as large as
    the activations themselves (what parity tests of the delta kernels need in order to see the delta)."""
    g = generator(seed + 2000003, device)
    x1 = randn_bf16((B, N, D), g)
    x2 = randn_bf16((B, N, D), g) if independent else perturb_all(x1, g)
    return x1, x2


def mlp_score_source(prev, seed):
    """prev [R,F] float32 -> cur = prev + hot/cold noise (float32), and the hot mask."""
    g = generator(seed + 3000003, prev.device)
    F = prev.shape[-1]
    hot = hot_mask(F, g)
    sigma = torch.where(hot, HOT_SIGMA, COLD_SIGMA).to(torch.float32)
    noise = torch.randn(prev.shape, generator=g, device=prev.device, dtype=torch.float32)
    return prev + sigma * noise, hot


def uniform_indices(R, C, k, seed, device="cpu", k_stride=None):
    """k distinct columns per row drawn uniformly, ascending: idx [R,k_stride] int32, counts [R]."""
    g = generator(seed + 4000003, device)
    k_stride = k if k_stride is None else k_stride
    idx = torch.zeros((R, k_stride), dtype=torch.int32, device=device)
    rows_per = max(1, (1 << 26) // max(C, 1))
    for r0 in range(0, R, rows_per):
        r1 = min(R, r0 + rows_per)
        keys = torch.rand((r1 - r0, C), generator=g, device=device)
        sel = keys.argsort(dim=1, stable=True)[:, :k].sort(dim=1).values
        idx[r0:r1, :k] = sel.to(torch.int32)
    counts = torch.full((R,), k, dtype=torch.int32, device=device)
    return idx, counts


def distinct_scores(R, C, seed, device="cpu"):
    """[R,C] float32 with no two equal entries in a row (a shuffled arithmetic grid plus jitter)."""
    g = generator(seed + 5000003, device)
    keys = torch.rand((R, C), generator=g, device=device)
    rank = keys.argsort(dim=1, stable=True).argsort(dim=1, stable=True).to(torch.float32)
    return (rank - (C - 1) / 2.0) / 64.0


# ---- bf16 storage format helpers (host side) --------------------------------

def np_f32(t):
    """torch tensor (any float dtype) -> contiguous float32 numpy array on the host."""
    return np.ascontiguousarray(t.detach().float().cpu().numpy())


def np_bf16_round(a):
    """float array -> float32 array whose values are exactly representable in bf16 (RNE)."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).float().numpy()


def stack_inputs(cfg, n_blocks, n_steps, seed, device="cpu", x_sigma=COLD_SIGMA):
    """Inputs of a stack of DiT blocks over consecutive diffusion steps.

    Returns blocks[b] = dict(q, k, v, x: lists over steps of bf16 tensors; w1, b1, w2, b2).  Every block has its
    own draws; step t+1 is step t perturbed by the recipe above with the block's fixed set of hot key tokens
    (x_sigma: the perturbation of the MLP input; parity tests raise it so that the MLP delta is not small).
    The blocks' inputs are independent of each other's outputs: projections and modulation between blocks are
    dense operations outside the method and are not modelled.
    """
    B, H, E, D, F = cfg["B"], cfg["H"], cfg["E"], cfg["D"], cfg["F"]
    N = config_tokens(cfg)
    blocks = []
    for b in range(n_blocks):
        g = generator(seed + 7919 * (b + 1), device)
        q = [randn_bf16((B, H, N, E), g)]
        k = [randn_bf16((B, H, N, E), g)]
        v = [randn_bf16((B, H, N, E), g)]
        x = [randn_bf16((B, N, D), g)]
        hot = hot_mask(N, g)
        for _ in range(1, n_steps):
            k.append(perturb_rows(k[-1], hot, g))
            v.append(perturb_rows(v[-1], hot, g))
            q.append(perturb_all(q[-1], g))
            x.append(perturb_all(x[-1], g, x_sigma))
        w1, b1, w2, b2 = mlp_weights(D, F, seed + 7919 * (b + 1), device)
        blocks.append(dict(q=q, k=k, v=v, x=x, w1=w1, b1=b1, w2=w2, b2=b2))
    return blocks


def block_indices(R, C, k, block, seed, device="cpu"):
    """k columns per row as whole runs of `block` consecutive, block-aligned columns drawn uniformly (the last run is
    cut so that exactly k columns remain), ascending: idx [R, k] int32, counts [R].  Stands for a [c, block]
    block-sparse pattern expressed as a column list."""
    g = generator(seed + 5000003, device)
    n_blocks_total = -(-C // block)
    n_pick = min(n_blocks_total, -(-k // block) + 1)
    keys = torch.rand((R, n_blocks_total), generator=g, device=device)
    picked = keys.argsort(dim=1, stable=True)[:, :n_pick].sort(dim=1).values                      # [R, n_pick] block numbers
    cols = (picked.unsqueeze(-1) * block + torch.arange(block, device=device)).reshape(R, -1)
    cols = torch.where(cols < C, cols, torch.full_like(cols, C))                     # the last block may be ragged
    cols = cols.sort(dim=1).values[:, :k]
    assert int(cols.max()) < C, "not enough columns in the picked blocks"
    counts = torch.full((R,), k, dtype=torch.int32, device=device)
    return cols.to(torch.int32).contiguous(), counts
