#!/usr/bin/env python3
"""Benchmark of the DFSS attention forward pass on one MI355X.

One "step" = one call of ``dfss_attention`` (all stages of the hot path: SDDMM with the pruning
epilogue, softmax over kept scores, SpMM) over one batch of synthetic inputs.  Prints ONE JSON line.

The metric is quoted on a family of workloads (2:4 and 1:2, L = 384 .. 4096), so the default run times all
of them: the headline (``value``, ``config.workload``) is the longest sequence, ``long_L4096_2to4``, and
``extra.sweep`` holds the same figures for every other configuration.  ``--workload NAME`` makes another
workload the headline and ``--no-sweep`` times only that one.

  value           whole-path throughput in TFLOP/s, counting the algorithmic FLOPs of the sparse path:
                  3 * BH * L^2 * d per step (2 L^2 d dense QK^T + L^2 d SpMM).
  extra / sweep   per workload: ms per step and TFLOP/s of dfss_attention (one kernel), of the one-kernel
                  full-attention baseline, of the staged path (three kernels) and of the three-stage dense
                  baseline, both speedups (one kernel vs one kernel, staged vs three-stage), the stage kernels
                  with stage 1 priced against the MFMA peak and the HBM peak.
  roofline        the kernel of the headline step (dfss_attention is one kernel): algorithmic FLOPs /
                  measured launch duration against the dense bf16 MFMA peak.
  cpu_baseline    the CPU oracle timed on the host cores, on a bounded sample of heads (context only).

Protocol.  Inputs are resident in HBM before timing starts.  The steps rotate over enough independent
buffer sets that no step finds its inputs (or, for the multi-kernel paths, its workspace) in the 256 MB
last-level cache ("cold"; ``--warm`` keeps one set).  The K steps asked for with ``--steps`` are captured in
one HIP graph, R times over (the same K steps, R chosen so that the graph runs for at least 20 ms: a short
graph is dominated by the host work around its launch and by clock ramp-up, so K = 20 and K = 2000 would
disagree), and the graph is launched once between two HIP events recorded on the stream the kernels run on.
ms_per_step = elapsed / (K * R); R is reported as ``config.graph_replays``.

Workloads whose name ends in ``_f32`` run the paper's second precision (float data, 1:2); ``--products``
selects how their fp32 products are formed.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
MFMA_F32_PEAK_TFLOPS = 157.3    # dense fp32 MFMA (the workloads of the 4-byte mode)
LLC_BYTES = 256 << 20           # last-level (Infinity) cache; L2 is 8 x 4 MiB on top
MIN_TIMED_MS = 20.0

HEADLINE = "long_L4096_2to4"
SWEEP = ("bert_base_L384_2to4", "bert_base_L512_1to2", "long_L1024_2to4", "long_L2048_2to4", "long_L4096_2to4",
         "large_head_L2048_d128_2to4", "large_head_L2048_d128_1to2")

# HBM bytes per launch of the one-kernel path measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by
# what the same counter reads for a plain copy of known size; the summaries under profiles/ give the commands.  Looked
# up by workload; a workload without a summary reports null.
TRAFFIC_FROM_PROFILES = {
    # workload: (bytes per launch, summary file)
    "long_L4096_2to4": (50.46e6, "profiles/hbm_traffic_k_fused32.md"),
    "large_head_L2048_d128_2to4": (134.36e6, "profiles/hbm_traffic_k_fused32.md"),
    "bert_base_L384_2to4": (19.01e6, "profiles/hbm_traffic_k_fused32.md"),
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200, help="steps per captured graph (the graph is replayed until "
                                                           "the timed region lasts 20 ms)")
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=HEADLINE, help="the headline workload")
    ap.add_argument("--no-sweep", action="store_true", help="time the headline workload only")
    ap.add_argument("--warm", action="store_true", help="single buffer set (cache-resident)")
    ap.add_argument("--no-graph", action="store_true", help="launch steps directly instead of from a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--key-padding", action="store_true",
                    help="headline only: run the key-bias entry points on a padded batch (seeded lengths in [L/2, L])")
    ap.add_argument("--block-pattern", action="store_true",
                    help="headline only: run the block-masked entry points with a seeded window + global + random "
                         "pattern of 64 x 64 blocks (one-kernel paths only; FLOPs are counted on the kept blocks)")
    ap.add_argument("--causal", action="store_true",
                    help="headline only: run the causal entry points (query i sees keys 0 .. i; FLOPs are counted on "
                         "the visible half of the score matrix)")
    ap.add_argument("--general-mask", action="store_true",
                    help="headline only: run the entry points that take an additive mask [L, L] (a seeded relative-"
                         "position term, finite everywhere; 4 bytes of reads per score)")
    ap.add_argument("--backward", action="store_true",
                    help="headline only: also time dfss_attention_backward on the results of the three forward stages")
    ap.add_argument("--unpadded", type=int, default=0, metavar="LEN",
                    help="headline only: also time dfss_attention_ragged / dense_attention_fused_ragged on arrays of LEN "
                         "queries and keys (LEN <= L, a multiple of 4) next to the padded-and-masked call")
    ap.add_argument("--products", choices=("fp32", "bf16x3"), default="bf16x3",
                    help="float workloads only: exact fp32 products (DFSS_F32) or bfloat16 pieces on the bf16 matrix "
                         "pipe (DFSS_F32_BF16X3, the default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 64 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


class Timer:
    """Times K steps from a HIP graph that repeats them until the timed region is long enough."""

    def __init__(self, torch, K, W, use_graph):
        self.torch, self.K, self.W, self.use_graph = torch, K, W, use_graph

    def __call__(self, step_fn, K=None):
        """-> (ms per step, graph replays)."""
        torch = self.torch
        K = self.K if K is None else K
        for i in range(self.W):
            step_fn(i)
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        if not self.use_graph:
            e0.record()
            for i in range(K):
                step_fn(i)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / K, 1
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(K):
                step_fn(i)
        g.replay()                     # untimed: uploads the graph
        torch.cuda.synchronize()
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        once = max(e0.elapsed_time(e1), 1e-3)
        R = max(1, math.ceil(MIN_TIMED_MS / once))
        if R > 1:
            # a graph R times as long (the same K steps R times over) instead of R launches of the short one:
            # no launch gaps inside the timed region
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(R):
                    for i in range(K):
                        step_fn(i)
            g.replay()
            torch.cuda.synchronize()
        e0.record()                    # the bracket: synchronised before, one graph launch, synchronised after
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (K * R), R


def run_workload(name, args, timer, torch, dfss, synth, headline):
    """All timings of one workload -> (dict of figures, context for the headline's extras)."""
    from paper_2203_00091_amd import Shape
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[name]
    f32 = w.float32
    split = f32 and args.products == "bf16x3"
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M,
              (dfss.DFSS_F32_BF16X3 if split else dfss.DFSS_F32) if f32 else dfss.DFSS_BF16)
    esz = 4 if f32 else 2
    has_fused = (not f32) or split     # one-kernel paths: the 2-byte modes and, in the float mode, bf16x3 products
    BH, L, d = w.BH, w.L, w.d

    # ---- buffers: enough sets that a step's data is not in the last-level cache ---------------------------
    Qc, Kc, Vc = synth.make(w)
    ws_bytes = max(dfss.dfss_workspace_bytes(s), dfss.dense_workspace_bytes(s))
    qkvo_bytes = 4 * BH * L * d * esz
    if args.warm:
        nsets = nws = 1
    else:
        nsets = max(2, math.ceil(3 * LLC_BYTES / qkvo_bytes))          # what the one-kernel steps touch
        nws = max(2, math.ceil(3 * LLC_BYTES / (qkvo_bytes + ws_bytes)))  # the multi-kernel steps also touch a workspace
    sets = [dict(Q=Qc.to(dev), K=Kc.to(dev), V=Vc.to(dev),
                 O=torch.empty((BH, L, d), dtype=s.torch_dtype, device=dev)) for _ in range(nsets)]
    wss = [torch.empty(ws_bytes, dtype=torch.uint8, device=dev) for _ in range(nws)]
    torch.cuda.synchronize()

    bias = key_len = None
    if headline and args.key_padding:
        lengths = synth.padding_lengths(w.B, L, w.seed + 7)
        bias = synth.key_padding_bias(lengths, L).to(dev)
        key_len = lengths.to(torch.int32).to(dev)
    block_mask, density = None, 1.0
    if headline and args.block_pattern:
        bm = synth.block_pattern(L // 64, L // 64, seed=w.seed + 9, window=1, n_global=1, n_random=2)
        density = float(bm.float().mean())
        block_mask = bm.to(dev)

    # block patterns: long row blocks shared between workgroups through a workspace where that measured faster
    # (2-byte data, d = 64, rows of 2048 keys and more)
    split_rows = block_mask is not None and not f32 and d == 64 and L >= 2048
    ws_split = (torch.empty(dfss.dfss_blocked_split_workspace_bytes(s), dtype=torch.uint8, device=dev)
                if split_rows else None)

    causal = bool(headline and args.causal)
    if causal:
        density = (L + 1) / (2.0 * L)      # visible entries of the score matrix

    gmask = None
    if headline and args.general_mask:
        gmask = synth.relative_position_mask(L, L, seed=w.seed + 11).to(dev)

    def step_sparse(i):
        b = sets[i % nsets]
        if gmask is not None:
            dfss.dfss_attention_mask(b["Q"], b["K"], b["V"], gmask, s, w.scale, O=b["O"])
        elif causal:
            dfss.dfss_attention_causal(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"])
        elif split_rows:
            dfss.dfss_attention_blocked_split(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"], ws=ws_split)
        elif block_mask is not None:
            dfss.dfss_attention_blocked(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"])
        elif has_fused:
            dfss.dfss_attention_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"])
        else:   # exact fp32 products: dfss_attention runs the three stages through a workspace
            dfss.dfss_attention(b["Q"], b["K"], b["V"], s, w.scale, O=b["O"], ws=wss[i % nws])

    def step_dense_fused(i):
        b = sets[i % nsets]
        if gmask is not None:
            dfss.dense_attention_fused_mask(b["Q"], b["K"], b["V"], gmask, s, w.scale, O=b["O"])
        elif causal:
            dfss.dense_attention_fused_causal(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"])
        elif split_rows:
            dfss.dense_attention_fused_blocked_split(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"],
                                                     ws=ws_split)
        elif block_mask is not None:
            dfss.dense_attention_fused_blocked(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"])
        else:
            dfss.dense_attention_fused_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"])

    def step_staged(i):
        b = sets[i % nsets]
        if gmask is not None:
            dfss.dfss_attention_staged_mask(b["Q"], b["K"], b["V"], gmask, s, w.scale, O=b["O"], ws=wss[i % nws])
            return
        fn = dfss.dfss_attention_staged_causal if causal else dfss.dfss_attention_staged_bias
        fn(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"], ws=wss[i % nws])

    def step_dense(i):
        b = sets[i % nsets]
        if gmask is not None:
            dfss.dense_attention_mask(b["Q"], b["K"], b["V"], gmask, s, w.scale, O=b["O"], ws=wss[i % nws])
            return
        fn = dfss.dense_attention_causal if causal else dfss.dense_attention_bias
        fn(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"], ws=wss[i % nws])

    n_vals, n_meta = dfss.dfss_vals_bytes(s), dfss.dfss_meta_bytes(s)
    meta_at = (n_vals + 255) // 256 * 256

    def stage_buffers(i):
        """The kept values and the metadata inside a workspace, where the staged call puts them."""
        ws = wss[i % nws]
        return ws[:n_vals].view(s.torch_dtype), ws[meta_at:meta_at + n_meta].view(torch.int16)

    def step_stage1(i):
        b = sets[i % nsets]
        vals, meta = stage_buffers(i)
        if gmask is not None:
            dfss.dfss_sddmm_prune_mask(b["Q"], b["K"], gmask, s, w.scale, vals=vals, meta=meta)
            return
        fn = dfss.dfss_sddmm_prune_causal if causal else dfss.dfss_sddmm_prune_bias
        fn(b["Q"], b["K"], bias, s, w.scale, vals=vals, meta=meta)

    def step_stage2(i):
        dfss.dfss_sparse_softmax(stage_buffers(i)[0], s)

    def step_stage3(i):
        b = sets[i % nsets]
        vals, meta = stage_buffers(i)
        dfss.dfss_spmm(vals, meta, b["V"], s, O=b["O"])

    def step_blocked_plain(i):   # the call without workspace, for comparison
        b = sets[i % nsets]
        dfss.dfss_attention_blocked(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"])

    # a padded batch given by its lengths instead of a bias array (2-byte data, no other mask)
    varlen = key_len is not None and not f32 and block_mask is None and not causal

    def step_varlen(i):
        b = sets[i % nsets]
        dfss.dfss_attention_varlen(b["Q"], b["K"], b["V"], key_len, s, w.scale, O=b["O"])

    blocked = block_mask is not None
    ms, replays = timer(step_sparse)
    ms_blocked_plain = timer(step_blocked_plain)[0] if split_rows else None
    ms_dense_fused = timer(step_dense_fused)[0] if has_fused else None
    if blocked:      # only the one-kernel paths take a block pattern
        ms_staged = ms_dense = k1 = k2 = k3 = None
    else:
        ms_staged = timer(step_staged)[0] if has_fused else ms
        ms_dense = timer(step_dense)[0]
        for i in range(nws):
            step_stage1(i)          # every workspace holds valid stage-1 output before stages 2, 3 run alone
        k1, k2, k3 = timer(step_stage1)[0], timer(step_stage2)[0], timer(step_stage3)[0]

    flops_alg = 3.0 * BH * L * L * d * density      # kept blocks only when a block pattern is given
    flops_eq = 4.0 * BH * L * L * d * density
    peak = MFMA_F32_PEAK_TFLOPS if f32 and not split else MFMA_BF16_PEAK_TFLOPS
    tflops = flops_alg / (ms * 1e-3) / 1e12
    res = {
        "workload": w.name, "B": w.B, "H": w.H, "L": L, "d": d, "N": w.N, "M": w.M,
        "dtype": "f32" if f32 else "bf16", "products": (args.products if f32 else "bf16"),
        "buffer_sets": nsets, "workspace_sets": nws,
        "dfss_attention_ms": round(ms, 5),
        "tflops_algorithmic": round(tflops, 2),
        "frac_of_mfma_peak": round(tflops / peak, 4),
        "dense_equivalent_tflops": round(flops_eq / (ms * 1e-3) / 1e12, 2),
        "dense_attention_fused_ms": None if ms_dense_fused is None else round(ms_dense_fused, 5),
        "speedup_vs_dense_attention_fused": None if ms_dense_fused is None else round(ms_dense_fused / ms, 4),
        "dfss_attention_staged_ms": None if ms_staged is None else round(ms_staged, 5),
        "dense_attention_3stage_ms": None if ms_dense is None else round(ms_dense, 5),
        "staged_speedup_vs_dense_attention_3stage": None if blocked else round(ms_dense / ms_staged, 4),
        "speedup_vs_dense_attention_3stage": None if blocked else round(ms_dense / ms, 4),
    }
    if varlen:
        res["key_lengths"] = [int(x) for x in lengths]
        res["dfss_attention_varlen_ms"] = round(timer(step_varlen)[0], 5)
        res["varlen_speedup_vs_dense_attention_fused"] = round(ms_dense_fused / res["dfss_attention_varlen_ms"], 4)
    if blocked:
        res["block_pattern_entry_points"] = ("dfss_attention_blocked_split / dense_attention_fused_blocked_split "
                                             "(main kernel + merge kernel per step)" if split_rows else
                                             "dfss_attention_blocked / dense_attention_fused_blocked")
        res["dfss_attention_blocked_without_workspace_ms"] = (None if ms_blocked_plain is None
                                                              else round(ms_blocked_plain, 5))
    if not blocked:
        # Algorithmic bytes per head: stage 1 reads Q, K = 4 L d and writes kept values L^2 plus metadata L^2 / 8;
        # stage 2 reads and writes L^2; stage 3 reads 1.125 L^2 + V and writes O (2-byte data; the 4-byte mode doubles all)
        bytes1 = BH * (2.0 * esz * L * d + (esz / 2 + esz / 16) * L * L)
        bytes2 = BH * (esz * L * L)
        bytes3 = BH * ((esz / 2 + esz / 16) * L * L + 2.0 * esz * L * d)
        flops1 = 2.0 * BH * L * L * d
        peak1 = MFMA_F32_PEAK_TFLOPS if f32 and not split else MFMA_BF16_PEAK_TFLOPS / (3.0 if f32 else 1.0)
        roof1 = min(peak1, HBM_PEAK_GBS * 1e9 * (flops1 / bytes1) / 1e12)
        kern = {"sddmm_prune": (k1, bytes1), "sparse_softmax": (k2, bytes2), "spmm": (k3, bytes3)}
        res.update({
            "stage_kernel_ms": {k: round(v[0], 5) for k, v in kern.items()},
            "stage_kernel_GBps": {k: round(v[1] / (v[0] * 1e-3) / 1e9, 1) for k, v in kern.items()},
            "stage_kernel_frac_of_hbm_peak": {k: round(v[1] / (v[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                              for k, v in kern.items()},
            "sddmm_prune_tflops": round(flops1 / (k1 * 1e-3) / 1e12, 2),
            "sddmm_prune_frac_of_mfma_peak": round(flops1 / (k1 * 1e-3) / 1e12 / peak, 4),
            # the lower of stage 1's two ceilings: the matrix peak (a third of the bf16 peak where every product is
            # three bf16 products), or the HBM peak times the stage's flops per algorithmic byte
            "sddmm_prune_roofline_tflops": round(roof1, 1),
            "sddmm_prune_frac_of_min_roofline": round(flops1 / (k1 * 1e-3) / 1e12 / roof1, 4),
        })
    ctx = dict(w=w, s=s, sets=sets, wss=wss, bias=bias, block_mask=block_mask, density=density, replays=replays,
               ms=ms, ms_staged=ms_staged, k1=k1, flops_alg=flops_alg, esz=esz, f32=f32, split=split,
               has_fused=has_fused, step_sparse=step_sparse, cpu=(Qc, Kc, Vc))
    return res, ctx


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only; --gpus N with N > 1 is not supported "
              "(heads are independent: the path would shard by splitting them across GPUs, with no exchange).",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2203_00091_amd as dfss
    from paper_2203_00091_amd import Shape, synth

    if not os.path.exists(dfss.library_path()):
        from paper_2203_00091_amd import build as b
        b.build()
    dfss.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.workload not in synth.WORKLOADS:
        print(f"bench.py: unknown workload {args.workload}", file=sys.stderr)
        sys.exit(2)
    wl = synth.WORKLOADS[args.workload]
    if args.general_mask and (wl.float32 or args.block_pattern or args.causal or args.key_padding or args.backward):
        print("bench.py: --general-mask runs the 2-byte workloads, forward pass, without the other mask flags",
              file=sys.stderr)
        sys.exit(2)
    if args.causal and (wl.float32 or args.block_pattern):
        print("bench.py: --causal runs the 2-byte workloads, without --block-pattern", file=sys.stderr)
        sys.exit(2)
    if wl.float32 and args.products == "fp32" and (args.backward or args.key_padding or args.block_pattern or args.unpadded):
        print("bench.py: with --products fp32 the float workloads run the plain forward pass only", file=sys.stderr)
        sys.exit(2)

    K, W = args.steps, args.warmup
    use_graph = not args.no_graph
    timer = Timer(torch, K, W, use_graph)

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # a short untimed run first: the first kernels of a process run at lower clocks
    warm_args = argparse.Namespace(**{**vars(args), "warm": True})
    run_workload("bert_base_L384_2to4", warm_args, Timer(torch, 20, 5, use_graph), torch, dfss, synth, headline=False)

    sweep = {}
    if not args.no_sweep:
        for name in SWEEP:
            if name == args.workload:
                continue
            sweep[name], ctx_other = run_workload(name, args, timer, torch, dfss, synth, headline=False)
            del ctx_other
            torch.cuda.empty_cache()
    head, ctx = run_workload(args.workload, args, timer, torch, dfss, synth, headline=True)
    if not args.no_sweep and args.workload in SWEEP and not (args.key_padding or args.block_pattern or args.causal
                                                             or args.general_mask):
        sweep[args.workload] = head
    w, s, sets = ctx["w"], ctx["s"], ctx["sets"]
    bias, block_mask = ctx["bias"], ctx["block_mask"]
    BH, L, d, esz = w.BH, w.L, w.d, ctx["esz"]
    f32, has_fused = ctx["f32"], ctx["has_fused"]
    ms = ctx["ms"]

    # launch cost seen from the host: the same steps launched one by one, no graph
    t0 = time.perf_counter()
    for i in range(K):
        ctx["step_sparse"](i)
    torch.cuda.synchronize()
    ms_direct = (time.perf_counter() - t0) / K * 1e3

    flops_alg = ctx["flops_alg"]
    plain = not (args.key_padding or args.block_pattern or args.causal or args.general_mask or f32)
    traffic = TRAFFIC_FROM_PROFILES.get(w.name) if plain else None
    if has_fused:
        # one kernel per step: the step time between the events IS the kernel's average launch duration
        roofline = {"bound": "mfma",
                    "kernel": ("k_fused_split (dfss_attention, float data, bf16x3 products)" if f32 else
                               "k_fused32 (dfss_attention, one kernel per step)" if plain else
                               "k_fused + k_merge_split (block pattern, long row blocks shared; two kernels per step)"
                               if head.get("block_pattern_entry_points", "").startswith("dfss_attention_blocked_split")
                               else "k_fused (the masked one-kernel path, one kernel per step)"),
                    "achieved": round(flops_alg / (ms * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(flops_alg / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                    "traffic": None if traffic is None else traffic[0],
                    "traffic_source": None if traffic is None else traffic[1],
                    "algorithmic_hbm_bytes_per_launch": (None if block_mask is not None else
                                                         4.0 * esz * BH * L * d + (4.0 * L * L if args.general_mask else 0.0)),
                    "avg_launch_ms": round(ms, 5), "algorithmic_flops_per_launch": flops_alg}
        if f32:   # every algorithmic product is executed as three bf16 products
            roofline["executed_matrix_flops_per_launch"] = 3.0 * flops_alg
    else:
        # exact fp32 products: three kernels per step; the score/prune kernel is the largest and is bound by the fp32
        # matrix instruction: 2 L^2 d flops per head per launch
        flops1 = 2.0 * BH * L * L * d
        k1 = ctx["k1"]
        roofline = {"bound": "mfma", "kernel": "k_scores_f32 (dfss_sddmm_prune, float data)",
                    "achieved": round(flops1 / (k1 * 1e-3) / 1e12, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(flops1 / (k1 * 1e-3) / 1e12 / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                    "algorithmic_hbm_bytes_per_launch": BH * (2.0 * esz * L * d + (esz / 2 + esz / 16) * L * L),
                    "avg_launch_ms": round(k1, 5), "algorithmic_flops_per_launch": flops1}

    extra = {k: v for k, v in head.items() if k not in ("workload", "B", "H", "L", "d", "N", "M", "dtype", "products")}
    extra["ms_per_step_direct_launch"] = round(ms_direct, 5)
    extra["sweep"] = sweep
    out = {
        "metric": "DFSS attention forward TFLOP/s (algorithmic 3*BH*L^2*d per step)",
        "value": round(flops_alg / (ms * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if f32 else "bf16",
        "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "L": L, "d": d, "N": w.N, "M": w.M,
                   "products": (args.products if f32 else "bf16"),
                   "key_padding": bool(args.key_padding), "causal": bool(args.causal),
                   "general_mask": bool(args.general_mask),
                   "block_pattern": (f"window +-1, 1 global, 2 random blocks of 64 x 64, density {ctx['density']:.3f}"
                                     if args.block_pattern else None),
                   "buffer_sets": head["buffer_sets"], "workspace_sets": head["workspace_sets"],
                   "cache": "warm" if args.warm else "cold (rotating buffer sets larger than the last-level cache)",
                   "launch": "hip graph of `steps` steps" if use_graph else "direct",
                   "graph_replays": ctx["replays"], "timed_steps": K * ctx["replays"],
                   "timer": "HIP events on the launch stream"},
        "roofline": roofline,
        "extra": extra,
    }

    if args.backward and block_mask is None:
        b = sets[0]
        vals = torch.empty((BH, L, s.Lc), dtype=s.torch_dtype, device=dev)
        meta = torch.empty((BH * L * s.meta_words,), dtype=torch.int16, device=dev)
        fn = dfss.dfss_sddmm_prune_causal if args.causal else dfss.dfss_sddmm_prune_bias
        fn(b["Q"], b["K"], bias, s, w.scale, vals=vals, meta=meta)
        dfss.dfss_sparse_softmax(vals, s)
        O_fwd = dfss.dfss_spmm(vals, meta, b["V"], s)
        dO = torch.randn(BH, L, d, device=dev).to(s.torch_dtype)
        grads = [torch.empty((BH, L, d), dtype=s.torch_dtype, device=dev) for _ in range(3)]
        ws_b = torch.empty(dfss.dfss_backward_workspace_bytes(s), dtype=torch.uint8, device=dev)

        def step_backward(i):
            dfss.dfss_attention_backward(dO, b["Q"], b["K"], b["V"], O_fwd, vals, meta, s, w.scale,
                                         dQ=grads[0], dK=grads[1], dV=grads[2], ws=ws_b)

        ms_bwd = timer(step_backward)[0]
        flops_bwd = 5.0 * BH * L * L * d      # dP: 2 L^2 d (formed densely), dQ, dK, dV: L^2 d each on kept entries
        out["extra"]["backward_ms_per_step"] = round(ms_bwd, 5)
        out["extra"]["backward_tflops"] = round(flops_bwd / (ms_bwd * 1e-3) / 1e12, 2)
        out["extra"]["backward_over_staged_forward"] = round(ms_bwd / ctx["ms_staged"], 3)

    if args.unpadded:
        Lr = args.unpadded
        if not (0 < Lr <= L and Lr % 4 == 0 and has_fused):
            print("bench.py: --unpadded LEN needs 0 < LEN <= L, LEN % 4 == 0 and a workload with a one-kernel path",
                  file=sys.stderr)
            sys.exit(2)
        b = sets[0]
        sr = Shape(w.B, w.H, Lr, Lr, d, w.N, w.M, s.dtype)
        Qr, Kr, Vr = (b[k][:, :Lr].contiguous() for k in ("Q", "K", "V"))
        Or = torch.empty((BH, Lr, d), dtype=s.torch_dtype, device=dev)
        pad_bias = torch.zeros((w.B, L), dtype=torch.float32, device=dev)
        pad_bias[:, Lr:] = float("-inf")
        t_r = timer(lambda i: dfss.dfss_attention_ragged(Qr, Kr, Vr, None, sr, w.scale, O=Or))[0]
        t_rd = timer(lambda i: dfss.dense_attention_fused_ragged(Qr, Kr, Vr, None, sr, w.scale, O=Or))[0]
        t_p = timer(lambda i: dfss.dfss_attention_bias(b["Q"], b["K"], b["V"], pad_bias, s, w.scale, O=b["O"]))[0]
        out["extra"]["unpadded"] = {
            "length": Lr, "cache": "warm (one buffer set)",
            "dfss_attention_ragged_ms_per_step": round(t_r, 5),
            "dense_attention_fused_ragged_ms_per_step": round(t_rd, 5),
            "padded_and_masked_dfss_attention_bias_ms_per_step": round(t_p, 5),
            "algorithmic_tflops": round(3.0 * BH * Lr * Lr * d / (t_r * 1e-3) / 1e12, 2)}
        if not f32:   # the stage calls take the same lengths (2-byte data)
            wsr = torch.empty(max(dfss.dfss_workspace_bytes(sr), dfss.dense_workspace_bytes(sr)), dtype=torch.uint8,
                              device=dev)
            t_s = timer(lambda i: dfss.dfss_attention_staged(Qr, Kr, Vr, sr, w.scale, O=Or, ws=wsr))[0]
            t_d3 = timer(lambda i: dfss.dense_attention(Qr, Kr, Vr, sr, w.scale, O=Or, ws=wsr))[0]
            t_sp = timer(lambda i: dfss.dfss_attention_staged(b["Q"], b["K"], b["V"], s, w.scale, O=b["O"], ws=ctx["wss"][0]))[0]
            out["extra"]["unpadded"].update({
                "dfss_attention_staged_ms_per_step": round(t_s, 5),
                "dense_attention_3stage_ms_per_step": round(t_d3, 5),
                "dfss_attention_staged_at_the_padded_length_ms_per_step": round(t_sp, 5)})

    if not args.no_cpu_baseline:
        import oracle
        Qc, Kc, Vc = ctx["cpu"]
        Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Qc, Kc, Vc))
        # bounded sample: as many heads as the host has threads (the oracle runs one head per thread), whole passes
        # for about ten seconds
        per_head_flops = 3.0 * L * L * d
        heads = int(max(1, min(BH, oracle.num_threads(), 4.0e10 // per_head_flops)))
        bm = None if block_mask is None else block_mask.cpu().numpy()
        oracle.attention(Qn[:1], Kn[:1], Vn[:1], w.N, w.M, w.scale, block_mask=bm)  # load + warm
        reps, dt = 0, 0.0
        t0 = time.perf_counter()
        while dt < 10.0 and reps < 500:
            oracle.attention(Qn[:heads], Kn[:heads], Vn[:heads], w.N, w.M, w.scale, block_mask=bm)
            reps += 1
            dt = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(reps * heads * per_head_flops * ctx["density"] / dt / 1e12, 6), "unit": "TFLOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{heads} of {BH} heads of {w.name}, {reps} passes in {dt:.2f} s"}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
