"""CPU-side checks of the C-ABI library: it loads, exports every symbol that
include/chipmunk.h declares, and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "chipmunk.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(chipmunk_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    import paper_2506_03275_amd as cm
    return cm.load()


def test_header_symbols_are_exported_and_bound(lib):
    import paper_2506_03275_amd as cm
    declared = _declared_symbols()
    assert len(declared) >= 11
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in chipmunk.h but not exported"
    assert sorted(cm.EXPORTED_SYMBOLS) == declared


def test_status_strings(lib):
    for code in range(0, -7, -1):
        text = lib.chipmunk_status_string(code).decode()
        assert text and text != "unknown status"
    assert lib.chipmunk_status_string(-99).decode() == "unknown status"


def test_bad_arguments_are_rejected_without_a_launch(lib):
    P = ctypes.c_void_p
    a = P(0x1000)   # never dereferenced: every call below must fail validation first
    # attention
    f = lib.chipmunk_attn_sparse_delta
    assert f(None, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -1
    assert f(a, a, a, a, None, a, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -1      # idx without counts
    assert f(a, a, a, a, a, a, a, 0, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -2
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 96, 192, 8, 0.1, 1.0, None) == -4           # E
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 64, 8, 0.1, 1.0, None) == -4           # c
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, -0.1, 1.0, None) == -2         # scale
    assert f(P(0x1008), a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -3  # alignment
    nan, inf = float("nan"), float("inf")
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, nan, 1.0, None) == -2          # NaN scale: nothing launched
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, inf, 1.0, None) == -2
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, 0.0, 1.0, None) == -2
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, 0.1, nan, None) == -2          # NaN o_scale
    assert f(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, 0.1, -inf, None) == -2
    # K/V rows are addressed with 32-bit byte offsets inside a head: N * E * 2 must stay below 2^32
    assert f(a, a, a, a, a, a, a, 1, 1, 1 << 24, 128, 192, 8, 0.1, 1.0, None) == -2
    assert f(a, a, a, a, a, a, a, 1, 1, 1 << 25, 64, 192, 8, 0.1, 1.0, None) == -2
    # block-sparse attention: the same checks as the column-list call
    fb = lib.chipmunk_attn_block_sparse_delta
    assert fb(a, a, a, None, a, a, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -1         # block list required
    assert fb(a, a, a, a, a, None, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -1         # base required
    assert fb(a, a, a, a, a, a, a, 1, 1, 128, 96, 192, 8, 0.1, 1.0, None) == -4             # E
    assert fb(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, -1, 0.1, 1.0, None) == -2           # kb_stride
    assert fb(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 1 << 25, 0.1, 1.0, None) == -2      # kb_stride * 128 overflows
    assert fb(a, a, a, a, a, a, a, 1, 1, 128, 128, 192, 8, float("nan"), 1.0, None) == -2
    assert fb(a, a, a, P(0x1002), a, a, a, 1, 1, 128, 128, 192, 8, 0.1, 1.0, None) == -3    # int32 alignment
    # bit-packed masks
    mi, im = lib.chipmunk_mask_to_indices, lib.chipmunk_indices_to_mask
    assert mi(None, 4, 1, 100, a, a, 8, None) == -1
    assert mi(a, 3, 1, 100, a, a, 8, None) == -2             # ld_words < ceil(C / 32)
    assert mi(a, 4, 1, 100, a, a, -1, None) == -2
    assert mi(P(0x1002), 4, 1, 100, a, a, 8, None) == -3
    assert im(a, a, 1, 100, 8, None, 4, None) == -1
    assert im(a, a, 1, (1 << 20) + 1, 8, a, 1 << 16, None) == -2   # longer than the row kept in LDS
    assert im(a, a, 0, 100, 8, a, 4, None) == -2
    # top-k
    t = lib.chipmunk_topk_cols
    assert t(None, None, 1, 8, 8, 2, a, a, 2, None) == -1
    assert t(a, None, 1, 8, 8, 9, a, a, 9, None) == -2      # k > C
    assert t(a, None, 1, 8, 8, 4, a, a, 3, None) == -2      # k_stride < k
    assert t(a, None, 1, 8, 6, 4, a, a, 4, None) == -2      # ld < C
    assert t(a, None, 1, 6, 6, 4, a, a, 4, None) == -3      # ld % 4
    # reorder
    r = lib.chipmunk_voxel_reorder
    assert r(None, None, None, None, 1, 0, 2, 2, 2, 0, 1, 1, 1, 4, 0, None) == -1
    assert r(a, None, None, None, 1, 0, 2, 2, 2, 0, 1, 1, 1, 4, 0, None) == -1
    assert r(None, None, a, None, 1, 0, 0, 2, 2, 0, 1, 1, 1, 4, 0, None) == -2
    assert r(a, P(0x100000), None, None, 1, 0, 2, 2, 2, 0, 1, 1, 1, 6, 0, None) == -3   # row_bytes % 4
    assert r(a, P(0x1010), None, None, 1, 0, 2, 2, 2, 0, 1, 1, 1, 16, 0, None) == -2    # overlap
    # MLP
    m = lib.chipmunk_mlp_sparse_delta
    assert m(a, a, None, a, a, a, a, 128, a, 1, 128, 256, 1024, 128, 16, 1, None, 0, None) == -5   # no workspace
    assert m(a, a, None, a, a, a, a, 128, a, 1, 128, 200, 1024, 128, 16, 1, a, 1 << 30, None) == -4  # D % 128
    assert m(a, a, None, a, a, a, a, 100, a, 1, 128, 256, 1024, 128, 16, 1, a, 1 << 30, None) == -2  # a_ld < N
    assert m(a, a, None, a, a, a, a, 132, a, 1, 128, 256, 1024, 128, 16, 1, a, 1 << 30, None) == -3  # a_ld % 8
    assert m(a, a, None, a, a, a, a, 128, a, 1, 128, 256, 1024, 128, 16, 7, a, 1 << 30, None) == -4  # act
    mo = lib.chipmunk_mlp_sparse_delta_overlapped
    assert lib.chipmunk_mlp_overlapped_workspace_bytes(1, 1024, 256, 1024, 128, 256) == 2 * 8 * 256 * 128 * 2
    assert mo(a, a, None, a, a, a, a, 128, a, 1, 128, 256, 1024, 128, 16, 1, a, 128 * 128 * 2, None) == -5   # one workspace is not enough
    assert mo(a, a, None, a, None, a, a, 128, a, 1, 128, 256, 1024, 128, 16, 1, a, 1 << 30, None) == -1
    assert lib.chipmunk_mlp_workspace_bytes(1, 1024, 256, 1024, 128, 256) == 8 * 256 * 128 * 2
    assert lib.chipmunk_mlp_workspace_bytes(1, 1024, 256, 1024, 100, 256) == 0
    d = lib.chipmunk_attn_dense
    assert d(a, a, a, a, a, 128, 1, 1, 128, 128, 192, 0.1, None, 0, None) == -5        # colsum needs ws
    assert d(a, a, a, a, a, 100, 1, 1, 128, 128, 192, 0.1, a, 1 << 20, None) == -2     # ld_colsum < N
    assert d(a, a, a, a, None, 0, 1, 1, 1 << 24, 128, 192, 0.1, None, 0, None) == -2   # N * E * 2 >= 2^32
    cs = lib.chipmunk_attn_colsum_stale
    assert cs(a, a, None, a, a, 128, 1, 1, 128, 128, 192, 0.1, None) == -1             # normalisers are required
    assert cs(a, a, a, a, a, 100, 1, 1, 128, 128, 192, 0.1, None) == -2                # ld_colsum < N
    assert cs(a, a, a, a, a, 128, 1, 1, 128, 96, 192, 0.1, None) == -4                 # E
    assert cs(a, a, P(0x1002), a, a, 128, 1, 1, 128, 128, 192, 0.1, None) == -3        # fp32 alignment
    assert cs(a, a, a, a, a, 1 << 24, 1, 1, 1 << 24, 128, 192, 0.1, None) == -2        # N * E * 2 >= 2^32
    assert cs(a, a, a, a, a, 128, 1, 1, 128, 128, 192, float("nan"), None) == -2
    fu = lib.chipmunk_attn_dense_colsum_stale
    assert fu(a, a, a, a, None, a, a, 128, None, None, 1, 1, 128, 128, 192, 0.1, None) == -1   # normalisers required
    assert fu(a, a, a, a, a, a, a, 128, a, None, 1, 1, 128, 128, 192, 0.1, None) == -1         # new_m without new_l
    assert fu(a, a, a, a, a, a, a, 100, None, None, 1, 1, 128, 128, 192, 0.1, None) == -2      # ld_colsum < N
    assert fu(a, a, a, a, a, a, a, 128, None, None, 1, 1, 128, 128, 160, 0.1, None) == -4      # c
    assert fu(a, a, a, a, a, a, a, 1 << 24, None, None, 1, 1, 1 << 24, 128, 192, 0.1, None) == -2   # N * E * 2 >= 2^32
    # the token-merged pre-activation: sizes the size query refuses are refused by the call as well
    tm = lib.chipmunk_mlp_tile_mean_preact
    assert lib.chipmunk_mlp_tile_mean_workspace_bytes(1, 1024, 256, 1024, 128) > 0
    assert lib.chipmunk_mlp_tile_mean_workspace_bytes(1, 1024, 200, 1024, 128) == 0
    assert lib.chipmunk_mlp_tile_mean_workspace_bytes(70000, 128, 128, 64, 128) > 0       # more chunks than one grid axis holds
    assert tm(a, a, a, 1, 1024, 256, 1024, 128, None, 0, None) == -5
    assert tm(a, a, a, 1, 1024, 256, 1024, 100, a, 1 << 30, None) == -4


def test_ceiling_probe_library_loads_and_rejects_bad_arguments():
    from paper_2506_03275_amd import ceilings
    lib = ceilings.load()
    text = open(os.path.join(ROOT, "paper_2506_03275_amd", "probe", "ceilings.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(chipmunk_probe_[a-z0-9_]+)\s*\(", text)))
    assert declared == ["chipmunk_probe_copy", "chipmunk_probe_mfma_bf16", "chipmunk_probe_mfma_flops",
                        "chipmunk_probe_read"]
    for name in declared:
        assert hasattr(lib, name)
    P = ctypes.c_void_p
    a = P(0x1000)
    assert lib.chipmunk_probe_mfma_flops(3, 10) == 0.0
    assert lib.chipmunk_probe_mfma_bf16(16, 1, 10, None, None) == -1
    assert lib.chipmunk_probe_mfma_bf16(24, 1, 10, a, None) == -1         # shape
    assert lib.chipmunk_probe_mfma_bf16(32, 3, 10, a, None) == -1         # workgroups per compute unit
    assert lib.chipmunk_probe_read(a, 24, a, None) == -1                  # bytes % 16
    assert lib.chipmunk_probe_copy(a, P(0x2008), 64, None) == -1          # alignment


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asked for more it says so and exits (no GPU is touched on the way)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
