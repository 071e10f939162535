#!/usr/bin/env python3
"""Benchmark of the Chipmunk hot path on one MI355X.

One "step" is one sparse-delta pass of a DiT block's attention + MLP over one
batch of synthetic tokens, every stage on the GPU through the C ABI:
  voxel reorder of the tokens -> top-k over the attention column sums ->
  column-sparse delta attention -> token-merged MLP scores -> top-k over
  |T - T_m| -> column-sparse delta MLP (GEMM1 + cache update, GEMM2 + merge).
The caches the step reads (column sums D, O_cache, A_cache, M_cache, T_m) come
from a dense step run once, untimed, with the library's dense kernels.

The headline `value` is useful TFLOP/s: the FLOPs of the selected (chunk, key
column) attention interactions and (chunk, hidden column) MLP interactions,
4*E*rows*count per attention unit and 4*D*rows*count per MLP unit, divided by
the whole step's time.  Softmax, GELU, index work and padding count as zero.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload hunyuan|flux|wan|tiny|stack]

The default workload is the HunyuanVideo-shaped configuration at 93 % column sparsity of attention and MLP: the
sparsity the headline metric is quoted at (the FLUX-shaped configuration keeps 10 % of the hidden columns, and the
paper's 9.3x kernel figure is for this sequence length).

prints ONE JSON line.  Nothing here runs on more than one GPU.
"""
import argparse
import hashlib
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synth_inputs as si  # noqa: E402

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0
CALIBRATION_COPY_BYTES = 256 << 20

# HBM-side bytes of one attn_sparse_delta_kernel launch (reads + writes beyond L2), from two
# `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then WRITE_SIZE), each counter scaled by what it
# read for the --traffic-calibration copy of known size; the summaries with the commands are
# profiles/attn_sparse_delta_traffic_<workload>.txt.  A counter run cannot happen inside this
# process, so the figure is carried here and reported with the live timing, but only while the
# attention kernel's sources are the ones the counters were taken on (ATTN_SOURCES_MEASURED is the
# digest attn_sources_digest() gave then); after any change to them `traffic` is null until the
# counters are taken again.
ATTN_SOURCES_MEASURED = "3b0c7ebaf0dd1455"
MEASURED_ATTN_TRAFFIC_BYTES = {   # read factor * FETCH_SIZE KiB + write factor * WRITE_SIZE KiB (mean of the last four launches of the counter runs)
    "flux": 2.0 * 66913 * 1024 + 1.0 * 27648 * 1024,
    "hunyuan": 2.0 * 12480026 * 1024 + 1.0 * 692736 * 1024,
    "wan": 2.0 * 9191464 * 1024 + 1.0 * 756001 * 1024,
}


def attn_sources_digest():
    """Digest of the sources the attention kernel is built from."""
    h = hashlib.sha256()
    for rel in ("paper_2506_03275_amd/csrc/attn.hip", "paper_2506_03275_amd/csrc/common.h"):
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_attn_traffic(workload, default_sparsity):
    if not default_sparsity or attn_sources_digest() != ATTN_SOURCES_MEASURED:
        return None
    return MEASURED_ATTN_TRAFFIC_BYTES.get(workload)

WORKLOAD_TEXT = {
    "tiny": "Tiny: 1024 tokens (8x8x16 grid), 2 heads x 64, MLP 256->1024, chunk 128, keep 25%",
    "flux": "FLUX.1-dev-shaped: 512 text + 4096 image tokens, 24 heads x 128, MLP 3072->12288, chunk 192, "
            "keep 7% of key columns and 10% of hidden columns",
    "hunyuan": "HunyuanVideo-shaped: 115200 video + 256 text tokens, 24 heads x 128, MLP 3072->12288, chunk 192, "
               "93% column sparsity",
    "wan": "WAN2.1-14B-shaped: 75600 video tokens, 40 heads x 128, MLP 5120->13824, chunk 192, 93% column sparsity",
    "stack": "Layer stack: 4 HunyuanVideo-shaped DiT blocks over 3 diffusion steps (step 1 dense, steps 2-3 column-sparse "
             "at 93%), MLP index work of the next block on a side stream",
}


class Timer:
    """HIP event pairs on the current stream (the stream the binding launches on)."""

    def __init__(self):
        self.spans = {}

    def span(self, name):
        start = torch.cuda.Event(enable_timing=True)
        stop = torch.cuda.Event(enable_timing=True)
        self.spans.setdefault(name, []).append((start, stop))
        return start, stop

    def mean_ms(self, name):
        spans = self.spans.get(name, [])
        if not spans:
            return None
        return sum(a.elapsed_time(b) for a, b in spans) / len(spans)


def build_state(cm, name, attn_keep, mlp_keep, seed, dev):
    cfg = si.CONFIGS[name]
    B, H, E, c, D, F = cfg["B"], cfg["H"], cfg["E"], cfg["c"], cfg["D"], cfg["F"]
    N = si.config_tokens(cfg)
    NB = -(-N // c)
    attn_keep = cfg["attn_keep"] if attn_keep is None else attn_keep
    mlp_keep = cfg["mlp_keep"] if mlp_keep is None else mlp_keep
    k_a, k_m = si.kept(N, attn_keep), si.kept(F, mlp_keep)
    st = dict(cfg=cfg, name=name, B=B, H=H, E=E, c=c, D=D, F=F, N=N, NB=NB, k_a=k_a, k_m=k_m,
              scale=1.0 / math.sqrt(E), act=cm.ACT_GELU_TANH)
    u8 = lambda n: torch.empty(max(int(n), 16), dtype=torch.uint8, device=dev)  # noqa: E731

    # ---- dense step (untimed): fills every cache the sparse step reads -------------------------
    (q1, k1, v1), (q2, k2, v2), _ = si.attn_steps(B, H, N, E, seed, dev)
    ld = -(-N // 4) * 4
    colsum = torch.empty((B, H, NB, ld), dtype=torch.float32, device=dev)
    o_dense = torch.empty_like(q1)
    cm.attn_dense(q1, k1, v1, o_dense, colsum, c, st["scale"], u8(cm.attn_dense_workspace_bytes(B, H, N)))
    idx_a = torch.zeros((B, H, NB, max(k_a, 1)), dtype=torch.int32, device=dev)
    cnt_a = torch.zeros((B, H, NB), dtype=torch.int32, device=dev)
    cm.load().chipmunk_topk_cols(colsum.data_ptr(), None, B * H * NB, N, ld, k_a, idx_a.data_ptr(), cnt_a.data_ptr(),
                                 idx_a.shape[-1], torch.cuda.current_stream().cuda_stream)
    o_cache_attn = torch.empty_like(q1)
    cm.attn_sparse_delta(q1, k1, v1, idx_a, cnt_a, o_dense, o_cache_attn, c, st["scale"], -1.0)
    del q1, k1, v1, o_dense

    w1, b1, w2, b2 = si.mlp_weights(D, F, seed, dev)
    x1, x2 = si.mlp_steps(B, N, D, seed, dev)
    # The MLP caches are updated in place, so a step repeated on the same input would find a_cache already equal
    # to its activations and multiply an all-zero delta in GEMM2.  Consecutive timed steps therefore alternate
    # between two inputs that differ like consecutive diffusion steps do: every step sees a non-zero delta.
    x3 = si.perturb_all(x2, si.generator(seed + 2000004, dev))
    a_cache = torch.zeros((B, F, -(-N // 8) * 8), dtype=torch.bfloat16, device=dev)
    m_cache = torch.empty_like(x1)
    cm.mlp_dense(x1, w1, b1, w2, b2, m_cache, a_cache, c, st["act"])
    T_m = torch.empty((B, NB, F), dtype=torch.float32, device=dev)
    ws_tm = u8(cm.mlp_tile_mean_workspace_bytes(B, N, D, F, c))
    cm.mlp_tile_mean_preact(x1, w1, T_m, c, ws_tm)
    del x1

    # the step's token input arrives in raster order; the step's first stage reorders it
    perm = torch.empty((N,), dtype=torch.int32, device=dev)
    npre, (gt, gh, gw), nsuf, (vt, vh, vw) = cfg["n_prefix"], cfg["grid"], cfg["n_suffix"], cfg["voxel"]
    cm.voxel_reorder(None, None, perm, None, npre, gt, gh, gw, nsuf, vt, vh, vw)
    x_rasters = []
    for xs in (x2, x3):
        x_raster = torch.empty_like(xs)
        cm.voxel_reorder(xs, x_raster, None, None, npre, gt, gh, gw, nsuf, vt, vh, vw, inverse=True)
        x_rasters.append(x_raster)
    torch.cuda.synchronize()

    st.update(q=q2, k=k2, v=v2, colsum=colsum, ld=ld, idx_a=idx_a, cnt_a=cnt_a, o_cache_attn=o_cache_attn,
              o_attn=torch.empty_like(q2), w1=w1, b1=b1, w2=w2, b2=b2, x_rasters=x_rasters, x=torch.empty_like(x2),
              x_expects=[x2, x3], step_count=0, a_cache=a_cache, m_cache=m_cache, T_m=T_m, T=torch.empty_like(T_m), ws_tm=ws_tm,
              idx_m=torch.zeros((B, NB, max(k_m, 1)), dtype=torch.int32, device=dev),
              cnt_m=torch.zeros((B, NB), dtype=torch.int32, device=dev),
              ws_mlp=u8(cm.mlp_workspace_bytes(B, N, D, F, c, max(k_m, 1))))
    return st


def sparse_step(cm, st, timer=None):
    """One pass of the whole hot path.  With a timer, every stage is bracketed by events."""
    cfg = st["cfg"]
    npre, (gt, gh, gw), nsuf, (vt, vh, vw) = cfg["n_prefix"], cfg["grid"], cfg["n_suffix"], cfg["voxel"]
    B, H, NB, N, F = st["B"], st["H"], st["NB"], st["N"], st["F"]
    lib = cm.load()
    stream = torch.cuda.current_stream().cuda_stream

    def stage(name, fn):
        if timer is None:
            fn()
            return
        a, b = timer.span(name)
        a.record()
        fn()
        b.record()

    which = st["step_count"] & 1                 # alternate between the two step inputs (see build_state)
    st["step_count"] += 1
    stage("voxel_reorder", lambda: cm.voxel_reorder(st["x_rasters"][which], st["x"], None, None, npre, gt, gh, gw,
                                                    nsuf, vt, vh, vw))
    stage("topk_attn", lambda: lib.chipmunk_topk_cols(st["colsum"].data_ptr(), None, B * H * NB, N, st["ld"],
                                                      st["k_a"], st["idx_a"].data_ptr(), st["cnt_a"].data_ptr(),
                                                      st["idx_a"].shape[-1], stream))
    stage("attn_sparse_delta", lambda: cm.attn_sparse_delta(st["q"], st["k"], st["v"], st["idx_a"], st["cnt_a"],
                                                            st["o_cache_attn"], st["o_attn"], st["c"], st["scale"],
                                                            1.0))
    stage("mlp_tile_mean_preact", lambda: cm.mlp_tile_mean_preact(st["x"], st["w1"], st["T"], st["c"], st["ws_tm"]))
    stage("topk_mlp", lambda: cm.topk_cols(st["T"].view(B * NB, F), st["T_m"].view(B * NB, F), st["k_m"],
                                           st["idx_m"].view(B * NB, -1), st["cnt_m"].view(-1)))
    stage("mlp_sparse_delta", lambda: cm.mlp_sparse_delta(st["x"], st["w1"], st["b1"], st["w2"], st["idx_m"],
                                                          st["cnt_m"], st["a_cache"], st["m_cache"], st["c"],
                                                          st["act"], st["ws_mlp"]))


def dense_step(cm, st, timer):
    out = st["o_attn"]
    a, b = timer.span("attn_dense")
    a.record()
    cm.attn_sparse_delta(st["q"], st["k"], st["v"], None, None, None, out, st["c"], st["scale"], 1.0)
    b.record()
    a, b = timer.span("mlp_dense")
    a.record()
    cm.mlp_dense(st["x"], st["w1"], st["b1"], st["w2"], st["b2"], st["dense_out"], st["dense_a"], st["c"], st["act"])
    b.record()


def useful_flops(st):
    rows_total = st["B"] * st["N"]
    attn = 4.0 * st["E"] * st["H"] * rows_total * st["k_a"]
    mlp = 4.0 * st["D"] * rows_total * st["k_m"]
    return attn, mlp


def cpu_baseline(st, budget_s=20.0):
    """The oracle, as it stands, on a bounded sample of the same step's units, on the host cores."""
    import oracle
    oracle.build()
    B, H, NB, N, E, c, D, F = (st[k] for k in ("B", "H", "NB", "N", "E", "c", "D", "F"))
    rng = np.random.default_rng(0)
    # attention units, each an independent (batch, head, chunk); cost 4*E*rows*k flops each
    per_unit = 4.0 * E * c * max(st["k_a"], 1)
    n_a = int(max(1, min(B * H * NB, (0.35 * budget_s * 4e9) // per_unit)))   # ~4 GFLOP/s assumed for sizing only
    units = [(int(rng.integers(B)), int(rng.integers(H)), int(rng.integers(NB))) for _ in range(n_a)]
    heads = sorted({(b, h) for b, h, _ in units})
    kv = {bh: (si.np_f32(st["k"][bh[0], bh[1]])[None, None], si.np_f32(st["v"][bh[0], bh[1]])[None, None])
          for bh in heads[:8]}
    units = [u for u in units if (u[0], u[1]) in kv]
    prepared = []
    for b, h, i in units:
        rows = slice(i * c, min(N, (i + 1) * c))
        prepared.append((si.np_f32(st["q"][b:b + 1, h:h + 1, rows]), kv[(b, h)][0], kv[(b, h)][1],
                         np.ascontiguousarray(st["idx_a"][b:b + 1, h:h + 1, i:i + 1].cpu().numpy()),
                         np.ascontiguousarray(st["cnt_a"][b:b + 1, h:h + 1, i:i + 1].cpu().numpy()),
                         si.np_f32(st["o_cache_attn"][b:b + 1, h:h + 1, rows]).astype(np.float64),
                         rows.stop - rows.start))
    t0 = time.perf_counter()
    fl_a = 0.0
    for qn, kn, vn, idxn, cntn, basen, nrows in prepared:
        oracle.attn_sparse_delta(qn, kn, vn, idxn, cntn, basen, c, st["scale"], 1.0)
        fl_a += 4.0 * E * nrows * float(cntn.sum())
    t_a = time.perf_counter() - t0
    # MLP units, each an independent (batch, chunk)
    per_unit = 4.0 * D * c * max(st["k_m"], 1)
    n_m = int(max(1, min(B * NB, (0.65 * budget_s * 4e9) // per_unit)))
    w1n, b1n, w2n = si.np_f32(st["w1"]), si.np_f32(st["b1"]), si.np_f32(st["w2"])
    chunks = sorted({(int(rng.integers(B)), int(rng.integers(NB))) for _ in range(n_m)})
    prepared = []
    for b, i in chunks:
        rows = slice(i * c, min(N, (i + 1) * c))
        prepared.append((si.np_f32(st["x"][b:b + 1, rows]),
                         np.ascontiguousarray(st["idx_m"][b:b + 1, i:i + 1].cpu().numpy()),
                         np.ascontiguousarray(st["cnt_m"][b:b + 1, i:i + 1].cpu().numpy()),
                         np.ascontiguousarray(si.np_f32(st["a_cache"][b:b + 1, :, rows]).astype(np.float64)),
                         np.ascontiguousarray(si.np_f32(st["m_cache"][b:b + 1, rows]).astype(np.float64)),
                         rows.stop - rows.start))
    t0 = time.perf_counter()
    fl_m = 0.0
    for xn, idxn, cntn, an, on, nrows in prepared:
        oracle.mlp_sparse_delta(xn, w1n, b1n, w2n, idxn, cntn, an, on, c, st["act"])
        fl_m += 4.0 * D * nrows * float(cntn.sum())
    t_m = time.perf_counter() - t0
    total_s = t_a + t_m
    return {
        "value": (fl_a + fl_m) / total_s / 1e12 if total_s > 0 else None,
        "unit": "TFLOP/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": f"{len(units)} of {B * H * NB} attention units ({t_a:.1f} s) + {len(chunks)} of {B * NB} MLP chunks "
                  f"({t_m:.1f} s) of this step, fp64 C oracle with OpenMP",
        "attn_tflops": fl_a / t_a / 1e12 if t_a > 0 else None,
        "mlp_tflops": fl_m / t_m / 1e12 if t_m > 0 else None,
    }


def library_context(st):
    """Dense attention and dense MLP of the same shape through torch's own kernels (whatever SDPA backend and GEMM
    library this build of torch picks): a second dense denominator beside this library's dense kernels.  A call that
    torch cannot run at this shape is reported as null with the reason."""
    import torch.nn.functional as F
    out = {"note": "torch " + torch.__version__ + "; not part of the library or of `value`"}
    rows = st["B"] * st["N"]

    def timed(fn, reps=2):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    try:
        from torch.nn.attention import SDPBackend, sdpa_kernel
        with sdpa_kernel([SDPBackend.FLASH_ATTENTION, SDPBackend.EFFICIENT_ATTENTION]):   # never the N x N fallback
            ms = timed(lambda: F.scaled_dot_product_attention(st["q"], st["k"], st["v"], scale=st["scale"]))
        out["sdpa_ms"] = ms
        out["sdpa_tflops"] = 4.0 * st["E"] * st["H"] * rows * st["N"] / (ms * 1e-3) / 1e12
    except Exception as e:  # noqa: BLE001 (context only: report and go on)
        out["sdpa_ms"] = None
        out["sdpa_error"] = f"{type(e).__name__}: {str(e)[:200]}"
    try:
        x, w1, b1, w2, b2 = st["x"], st["w1"], st["b1"], st["w2"], st["b2"]

        def mlp():
            h = F.gelu(F.linear(x, w1, b1), approximate="tanh")
            return torch.matmul(h, w2) + b2

        ms = timed(mlp)
        out["mlp_ms"] = ms
        out["mlp_tflops"] = 4.0 * st["D"] * rows * st["F"] / (ms * 1e-3) / 1e12
    except Exception as e:  # noqa: BLE001
        out["mlp_ms"] = None
        out["mlp_error"] = f"{type(e).__name__}: {str(e)[:200]}"
    return out


def stack_bench(cm, args, steps, warmup, dev):
    """The layer-stack workload: 4 HunyuanVideo-shaped blocks x 3 diffusion steps.  A timed "step" here is one pass of the
    two column-sparse diffusion steps over the four blocks (8 block passes), with the next block's MLP index work
    on a side stream; the serial schedule and the dense step are timed beside it."""
    from paper_2506_03275_amd import stack
    cfg = si.CONFIGS["hunyuan"]
    n_blocks, n_steps = 4, 3
    N = si.config_tokens(cfg)
    k_a = si.kept(N, cfg["attn_keep"] if args.attn_keep is None else args.attn_keep)
    k_m = si.kept(cfg["F"], cfg["mlp_keep"] if args.mlp_keep is None else args.mlp_keep)
    inputs = si.stack_inputs(cfg, n_blocks, n_steps, args.seed, dev)
    blocks = [stack.Block(inp, cfg["c"], k_a, k_m) for inp in inputs]

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / reps, a.elapsed_time(b) / reps

    def first_dense():                      # Alg. 2 with exact column sums (two passes over q k^T)
        for blk in blocks:
            blk.has_stats = False
        stack.dense_step(blocks, 0)

    _, dense_ms = timed(first_dense, 1)
    # a later dense step: column sums against the previous dense step's normalisers, inside the attention kernel (Alg. 4)
    _, refresh_ms = timed(lambda: stack.dense_step(blocks, 0), 1)
    side = torch.cuda.Stream()

    def sparse_pass(side_stream):
        for step in (1, 2):
            stack.sparse_step(blocks, step, side_stream)

    for _ in range(warmup):
        sparse_pass(side)
    serial_wall, serial_ms = timed(lambda: sparse_pass(None), steps)
    overlap_wall, overlap_ms = timed(lambda: sparse_pass(side), steps)

    rows = cfg["B"] * N
    fl_attn = 4.0 * cfg["E"] * cfg["H"] * rows * k_a
    fl_mlp = 4.0 * cfg["D"] * rows * k_m
    passes = n_blocks * (n_steps - 1)
    value = passes * (fl_attn + fl_mlp) / (overlap_wall * 1e-3) / 1e12
    # the dominant kernel, timed alone on the current stream
    blk = blocks[0]
    _, attn_ms = timed(lambda: blk.attn_delta(1), 5)
    achieved = fl_attn / (attn_ms * 1e-3) / 1e12
    line = {
        "metric": "sparse-delta attn+MLP useful TFLOP/s (whole step: reorder, top-k, scores, attention and MLP deltas)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": overlap_wall, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT["stack"], "name": "stack", "blocks": n_blocks, "diffusion_steps": n_steps,
                   "tokens": N, "attn_columns_kept": k_a, "mlp_columns_kept": k_m, "seed": args.seed,
                   "note": "one timed step = the two sparse diffusion steps over the four blocks; the token reorder "
                           "happens once per generation and is not part of a block pass; the blocks' inputs are "
                           "pre-generated, so overlapping the NEXT block's index work is a property of this stack"},
        "roofline": {"kernel": "attn_sparse_delta_kernel", "bound": "mfma", "achieved": achieved,
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                     "traffic": measured_attn_traffic("hunyuan", args.attn_keep is None),
                     "launch_ms": attn_ms, "algorithmic_flops_per_launch": fl_attn},
        "stack": {"sparse_pass_ms_side_stream": overlap_ms, "sparse_pass_ms_serial": serial_ms,
                  "side_stream_gain": serial_ms / overlap_ms, "dense_step_ms_4_blocks": dense_ms,
                  "dense_refresh_step_ms_4_blocks": refresh_ms,
                  "per_block_pass_ms": overlap_ms / passes},
    }
    print(json.dumps(line))


def ceilings_bench(dev):
    """What the device sustains for bare bf16 MFMA streams and for streaming reads and copies: the measured
    ceilings the roofline fractions are also quoted against."""
    from paper_2506_03275_amd import ceilings as cl
    sink = torch.zeros(1 << 20, dtype=torch.float32, device=dev)
    out = {"mfma_bf16_tflops": {}, "unit_note": "waves = waves per SIMD"}

    def timed(fn, reps=3):
        best = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return best

    iters = 60000                                    # 20-40 ms per launch: long enough for the clocks to settle
    for shape in (16, 32):
        for waves in (1, 2):
            ms = timed(lambda: cl.mfma_bf16(shape, waves, iters // waves, sink))
            name = f"{shape}x{shape}x{512 // shape}_waves{waves}"
            out["mfma_bf16_tflops"][name] = round(cl.mfma_flops(waves, iters // waves) / (ms * 1e-3) / 1e12, 1)
    src = torch.ones(1 << 28, dtype=torch.float32, device=dev)        # 1 GiB
    dst = torch.empty_like(src)
    nbytes = src.numel() * 4
    out["read_GBps"] = round(nbytes / (timed(lambda: cl.read(src, sink), 5) * 1e-3) / 1e9, 1)
    out["copy_GBps_read_plus_write"] = round(2 * nbytes / (timed(lambda: cl.copy(src, dst), 5) * 1e-3) / 1e9, 1)
    assert torch.equal(dst[:4096], src[:4096]) and torch.equal(dst[-4096:], src[-4096:])
    print(json.dumps({"ceilings": out}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="hunyuan", choices=sorted(si.CONFIGS) + ["stack"])
    ap.add_argument("--attn-keep", type=float, default=None, help="fraction of key columns kept (default: the config's)")
    ap.add_argument("--mlp-keep", type=float, default=None, help="fraction of hidden columns kept")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--library-context", action="store_true",
                    help="also time torch's own dense attention (SDPA) and dense MLP (matmul) at the same shape: "
                         "context for the dense denominator, never used by the library or by `value`")
    ap.add_argument("--index-structures", action="store_true",
                    help="also time the attention kernel alone on two other index structures of the same size: "
                         "columns drawn uniformly per chunk, and whole blocks of 128 consecutive columns")
    ap.add_argument("--mlp-overlap", action="store_true",
                    help="also time the MLP delta with the cache write-back inside the second GEMM's launch "
                         "(chipmunk_mlp_sparse_delta_overlapped) beside the plain call")
    ap.add_argument("--graph", action="store_true",
                    help="also time the step captured as one HIP graph (reported beside the eager numbers)")
    ap.add_argument("--ceilings", action="store_true",
                    help="print what the device sustains for bare MFMA streams and streaming reads/copies, and exit")
    ap.add_argument("--traffic-calibration", action="store_true",
                    help="also launch a plain elementwise copy of 256 MiB (untimed), the known-size kernel that "
                         "scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path has no collectives: every (batch, head, chunk) "
              "unit is independent and would shard without exchange). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback.", file=sys.stderr)
        sys.exit(2)
    big = args.workload in ("hunyuan", "wan", "stack")
    steps = args.steps if args.steps is not None else (5 if big else 50)
    warmup = args.warmup if args.warmup is not None else (1 if big else 5)

    import paper_2506_03275_amd as cm
    cm.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.ceilings:
        ceilings_bench(dev)
        return
    if args.workload == "stack":
        stack_bench(cm, args, steps, warmup, dev)
        return
    st = build_state(cm, args.workload, args.attn_keep, args.mlp_keep, args.seed, dev)

    if args.traffic_calibration:
        src = torch.ones(CALIBRATION_COPY_BYTES // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)   # reads and writes CALIBRATION_COPY_BYTES each
        torch.cuda.synchronize()
        del src, dst

    for _ in range(warmup):
        sparse_step(cm, st)
    torch.cuda.synchronize()
    timer = Timer()
    t0 = time.perf_counter()
    for _ in range(steps):
        sparse_step(cm, st, timer)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / steps
    assert torch.equal(st["x"], st["x_expects"][(st["step_count"] - 1) & 1]), "voxel reorder did not restore the token order"
    delta_rms = float(st["ws_mlp"][: 1 << 20].view(torch.bfloat16).float().pow(2).mean().sqrt())
    assert st["k_m"] == 0 or delta_rms > 0.0, "the timed MLP steps multiplied an all-zero delta"

    stages = {n: timer.mean_ms(n) for n in timer.spans}
    fl_attn, fl_mlp = useful_flops(st)
    value = (fl_attn + fl_mlp) / (ms_per_step * 1e-3) / 1e12

    # dominant kernel: the column-sparse attention kernel (one launch per step)
    attn_ms = stages["attn_sparse_delta"]
    achieved = fl_attn / (attn_ms * 1e-3) / 1e12
    roofline = {"kernel": "attn_sparse_delta_kernel", "bound": "mfma", "achieved": achieved,
                "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": measured_attn_traffic(args.workload, args.attn_keep is None),
                "launch_ms": attn_ms, "algorithmic_flops_per_launch": fl_attn}

    graph_extra = None
    if args.graph:
        # The same step as one HIP graph per step input (the two inputs alternate as in the eager loop): no launch
        # gaps and no per-stage events between the kernels.
        graphs = []
        for which in (0, 1):
            st["step_count"] = which
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                sparse_step(cm, st)
            graphs.append(g)
        for i in range(2 * max(warmup, 1)):
            graphs[i & 1].replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            graphs[i & 1].replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / steps
        assert any(torch.equal(st["x"], e) for e in st["x_expects"]), "voxel reorder did not restore the token order (graph replay)"
        graph_extra = {"ms_per_step": g_ms, "useful_tflops": (fl_attn + fl_mlp) / (g_ms * 1e-3) / 1e12}

    extra = {"stage_ms": stages,
             "attn_useful_tflops": achieved,
             "mlp_useful_tflops": fl_mlp / (stages["mlp_sparse_delta"] * 1e-3) / 1e12}
    if graph_extra is not None:
        extra["hip_graph"] = graph_extra
    if args.index_structures:
        R = st["B"] * st["H"] * st["NB"]
        kinds = {"topk_of_column_sums": (st["idx_a"], st["cnt_a"])}
        iu, cu = si.uniform_indices(R, st["N"], st["k_a"], args.seed, dev)
        kinds["uniform_per_chunk"] = (iu.view(st["B"], st["H"], st["NB"], -1), cu.view(st["B"], st["H"], st["NB"]))
        ib, cb = si.block_indices(R, st["N"], st["k_a"], 128, args.seed, dev)
        kinds["blocks_of_128_columns"] = (ib.view(st["B"], st["H"], st["NB"], -1), cb.view(st["B"], st["H"], st["NB"]))
        extra["attn_index_structures"] = {}

        def time_launch(fn):
            t = Timer()
            for i in range(4):
                a, b = t.span("k") if i else Timer().span("warm")
                a.record()
                fn()
                b.record()
            torch.cuda.synchronize()
            return t.mean_ms("k")

        for kind, (idx, cnt) in kinds.items():
            ms = time_launch(lambda: cm.attn_sparse_delta(st["q"], st["k"], st["v"], idx, cnt, st["o_cache_attn"],
                                                          st["o_attn"], st["c"], st["scale"], 1.0))
            extra["attn_index_structures"][kind] = {"ms": ms, "useful_tflops": fl_attn / (ms * 1e-3) / 1e12}
        # the [c, 128] block pattern of Table 2 on the kernel that walks block lists (no per-column index), beside
        # the column kernel on a list of the same length
        n_blocks = max(1, st["k_a"] // cm.ATTN_BLOCK_COLUMNS)
        kept = n_blocks * cm.ATTN_BLOCK_COLUMNS
        keys = torch.rand((R, -(-st["N"] // cm.ATTN_BLOCK_COLUMNS)), device=dev, generator=si.generator(args.seed + 17, dev))
        blocks = keys.argsort(dim=1)[:, :n_blocks].sort(dim=1).values.to(torch.int32).contiguous()
        bcnt = torch.full((R,), n_blocks, dtype=torch.int32, device=dev)
        fl_blocks = 4.0 * st["E"] * st["H"] * st["B"] * st["N"] * kept      # upper bound: the last block may be cut at N
        ms = time_launch(lambda: cm.attn_block_sparse_delta(st["q"], st["k"], st["v"],
                                                            blocks.view(st["B"], st["H"], st["NB"], -1),
                                                            bcnt.view(st["B"], st["H"], st["NB"]), st["o_cache_attn"],
                                                            st["o_attn"], st["c"], st["scale"], 1.0))
        extra["attn_index_structures"]["block_list_kernel_c_x_128"] = {
            "ms": ms, "blocks_per_chunk": n_blocks, "columns_kept": kept, "useful_tflops": fl_blocks / (ms * 1e-3) / 1e12}
        iu2, cu2 = si.uniform_indices(R, st["N"], kept, args.seed + 1, dev)
        ms = time_launch(lambda: cm.attn_sparse_delta(st["q"], st["k"], st["v"], iu2.view(st["B"], st["H"], st["NB"], -1),
                                                      cu2.view(st["B"], st["H"], st["NB"]), st["o_cache_attn"], st["o_attn"],
                                                      st["c"], st["scale"], 1.0))
        extra["attn_index_structures"]["column_kernel_same_count_uniform"] = {
            "ms": ms, "columns_kept": kept, "useful_tflops": fl_blocks / (ms * 1e-3) / 1e12}
        del blocks, iu2
        del kinds, iu, ib

    if args.mlp_overlap:
        # same indices, the two step inputs alternating so that the deltas are not zero; plain and overlapped in turn
        ws2 = torch.empty(max(cm.mlp_overlapped_workspace_bytes(st["B"], st["N"], st["D"], st["F"], st["c"], max(st["k_m"], 1)), 16),
                          dtype=torch.uint8, device=dev)
        t = Timer()
        for i in range(12):
            x_in = st["x_expects"][i & 1]
            for name, fn, w in (("plain", cm.mlp_sparse_delta, st["ws_mlp"]), ("overlapped", cm.mlp_sparse_delta_overlapped, ws2)):
                a, b = t.span(name) if i >= 2 else Timer().span("warm")
                a.record()
                fn(x_in, st["w1"], st["b1"], st["w2"], st["idx_m"], st["cnt_m"], st["a_cache"], st["m_cache"], st["c"],
                   st["act"], w)
                b.record()
        torch.cuda.synchronize()
        extra["mlp_writeback_overlap"] = {"plain_ms": t.mean_ms("plain"), "overlapped_ms": t.mean_ms("overlapped")}
        del ws2

    if not args.no_dense:
        st["dense_out"] = torch.empty_like(st["x"])
        st["dense_a"] = torch.empty_like(st["a_cache"])
        dt = Timer()
        n_dense = 2 if big else 10
        dense_step(cm, st, Timer())
        for _ in range(n_dense):
            dense_step(cm, st, dt)
        torch.cuda.synchronize()
        d_attn, d_mlp = dt.mean_ms("attn_dense"), dt.mean_ms("mlp_dense")
        rows_total = st["B"] * st["N"]
        extra["dense"] = {"attn_ms": d_attn, "mlp_ms": d_mlp,
                          "attn_tflops": 4.0 * st["E"] * st["H"] * rows_total * st["N"] / (d_attn * 1e-3) / 1e12,
                          "mlp_tflops": 4.0 * st["D"] * rows_total * st["F"] / (d_mlp * 1e-3) / 1e12}
        extra["speedup_vs_dense"] = {
            "attn_kernel": d_attn / attn_ms,
            "mlp_kernels": d_mlp / stages["mlp_sparse_delta"],
            "attn_plus_mlp_kernels": (d_attn + d_mlp) / (attn_ms + stages["mlp_sparse_delta"]),
            "whole_step": (d_attn + d_mlp) / ms_per_step,
        }
        del st["dense_out"], st["dense_a"]

    if args.library_context:
        ctx = library_context(st)
        if "dense" in extra:   # the speedups again, against the faster dense implementation of each op
            best_attn = min(x for x in (extra["dense"]["attn_ms"], ctx.get("sdpa_ms")) if x)
            best_mlp = min(x for x in (extra["dense"]["mlp_ms"], ctx.get("mlp_ms")) if x)
            ctx["speedup_vs_faster_dense"] = {
                "attn_kernel": best_attn / attn_ms,
                "mlp_kernels": best_mlp / stages["mlp_sparse_delta"],
                "attn_plus_mlp_kernels": (best_attn + best_mlp) / (attn_ms + stages["mlp_sparse_delta"]),
                "whole_step": (best_attn + best_mlp) / ms_per_step,
            }
        extra["library_context"] = ctx

    line = {
        "metric": "sparse-delta attn+MLP useful TFLOP/s (whole step: reorder, top-k, scores, attention and MLP deltas)",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": WORKLOAD_TEXT[args.workload], "name": args.workload, "tokens": st["N"],
                   "attn_columns_kept": st["k_a"], "mlp_columns_kept": st["k_m"],
                   "attn_sparsity": 1.0 - st["k_a"] / st["N"], "mlp_sparsity": 1.0 - st["k_m"] / st["F"],
                   "seed": args.seed},
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(st)
    line.update(extra)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
