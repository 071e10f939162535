"""The entry point that allocates nothing (chipmunk_mlp_tile_mean_preact_static) against the general one, called
through the C ABI: two calls in a row on the library's fixed scratch array, the second on a smaller input, and a
problem beyond the array's capacity."""
import ctypes

import numpy as np
import pytest
import torch

import synth_inputs as si
from parity import SCORE_TOL, rel_err

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _scores_both_ways(lib, B, N, D, F, c, seed):
    g = si.generator(seed, DEV)
    x = si.randn_bf16((B, N, D), g)
    w1 = si.randn_bf16((F, D), g, 1.0 / np.sqrt(D))
    NB = -(-N // c)
    need = lib.chipmunk_mlp_tile_mean_workspace_bytes(B, N, D, F, c)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    T_ref = torch.full((B, NB, F), float("nan"), dtype=torch.float32, device=DEV)
    T_new = torch.full((B, NB, F), float("nan"), dtype=torch.float32, device=DEV)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    assert lib.chipmunk_mlp_tile_mean_preact(x.data_ptr(), w1.data_ptr(), T_ref.data_ptr(), B, N, D, F, c,
                                             ws.data_ptr(), need, stream) == 0
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    assert lib.chipmunk_mlp_tile_mean_preact_static(x.data_ptr(), w1.data_ptr(), T_new.data_ptr(), B, N, D, F, c,
                                                    stream) == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    return x, w1, T_ref, T_new


def test_static_scratch_entry_point_matches_the_general_one(oracle):
    import paper_2506_03275_amd as cm
    lib = cm.load()
    assert lib.chipmunk_mlp_tile_mean_preact_static_capacity() == 32 << 20
    # first call: many chunks, the contraction cut in pieces; second call, right after it on the same array: smaller
    for (B, N, D, F, c), seed in (((2, 150 * 192 - 50, 256, 320, 192), 3), ((1, 1000, 128, 192, 128), 4)):
        x, w1, T_ref, T_new = _scores_both_ways(lib, B, N, D, F, c, seed)
        assert bool(torch.isfinite(T_new).all())
        assert rel_err(T_new.cpu().numpy(), T_ref.cpu().numpy().astype(np.float64)) <= 1e-5
        assert rel_err(T_new.cpu().numpy(), oracle.mlp_tile_scores(si.np_f32(x), si.np_f32(w1), c)) <= SCORE_TOL
    # the HunyuanVideo-shaped problem: the general workspace (66 MB) exceeds the array, fewer pieces fit it
    cfg = si.CONFIGS["hunyuan"]
    B, D, F, c = cfg["B"], cfg["D"], cfg["F"], cfg["c"]
    N = si.config_tokens(cfg)
    assert lib.chipmunk_mlp_tile_mean_workspace_bytes(B, N, D, F, c) > (32 << 20)
    x, w1, T_ref, T_new = _scores_both_ways(lib, B, N, D, F, c, 5)
    assert rel_err(T_new.cpu().numpy(), T_ref.cpu().numpy().astype(np.float64)) <= 1e-5
    # beyond the capacity: 3000 chunks of means at D = 3072 are 36.9 MB; refused before any launch
    a = ctypes.c_void_p(0x1000)
    assert lib.chipmunk_mlp_tile_mean_preact_static(a, a, a, 1, 3000 * 192, 3072, 64, 192, None) == -5
    assert lib.chipmunk_mlp_tile_mean_preact_static(None, a, a, 1, 1024, 256, 1024, 128, None) == -1
    assert lib.chipmunk_mlp_tile_mean_preact_static(a, a, a, 1, 1024, 200, 1024, 128, None) == -4
