#!/usr/bin/env python3
"""Benchmark of the DFSS attention forward pass on one MI355X.

One "step" = one call of ``dfss_attention`` (all stages of the hot path: SDDMM with the
pruning epilogue, softmax over kept scores, SpMM) over one batch of synthetic inputs of
the named workload.  Prints ONE JSON line.

  value           whole-path throughput in TFLOP/s, counting the algorithmic FLOPs of the
                  sparse path: 3 * BH * L^2 * d per step (2 L^2 d dense QK^T + L^2 d SpMM).
  extra           the same step for ``dense_attention`` on the same GPU, the speedup, the
                  dense-equivalent rate (4 * BH * L^2 * d), warm-cache figures.
  roofline        the kernel of the step (dfss_attention is one fused kernel): algorithmic
                  FLOPs / measured launch duration against the dense bf16 MFMA peak.
  cpu_baseline    the CPU oracle timed on the host cores (context only).

Workloads whose name ends in ``_f32`` run the paper's second precision (float data, 1:2).  With the
default ``--products bf16x3`` (fp32 products formed from bfloat16 pieces on the bf16 matrix pipe)
everything is as for the 2-byte workloads (``dfss_attention`` is one kernel).  With ``--products fp32``
``dfss_attention`` is the three stage kernels, the only full-attention baseline is the three-stage
``dense_attention``, and the roofline object describes the score/prune kernel (the largest of the
three) against the fp32 MFMA peak.

Inputs are resident in HBM before timing starts.  By default the steps rotate over enough
independent buffer sets that no step finds its inputs or workspace in the last-level cache
(``--warm`` keeps one set).  The K timed steps are captured in one HIP graph and replayed
once between two device synchronisations, so host launch cost is not part of the figure.
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
# HBM bytes per launch of the fused kernel, measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# (scaled by what the same counters read for a plain 64 MiB copy); summaries under profiles/.
MEASURED_TRAFFIC_BYTES = {"bert_base_L384_2to4": 14.23e6 + 4.72e6,
                          "bert_base_L512_1to2_f32": 75.6e6 + 25.2e6}   # (one-kernel path, bf16x3 products)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the timed bracket (synchronise, replay the graph of K steps, synchronise) contains about 0.4 ms of host work
    # for launching the graph and noticing its end: K = 2000 keeps that below 2 % of a 12 us step
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="bert_base_L384_2to4")
    ap.add_argument("--warm", action="store_true", help="single buffer set (cache-resident)")
    ap.add_argument("--no-graph", action="store_true", help="launch steps directly instead of one HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--key-padding", action="store_true",
                    help="run the key-bias entry points on a padded batch (seeded lengths in [L/2, L])")
    ap.add_argument("--block-pattern", action="store_true",
                    help="run the block-masked entry points with a seeded window + global + random pattern of "
                         "64 x 64 blocks (fused kernels only; FLOPs are counted on the kept blocks)")
    ap.add_argument("--backward", action="store_true",
                    help="also time dfss_attention_backward (gradients through the fixed selection) on the "
                         "results of the three forward stages; reported under extra")
    ap.add_argument("--unpadded", type=int, default=0, metavar="LEN",
                    help="also time dfss_attention_ragged / dense_attention_fused_ragged on arrays of LEN queries and "
                         "keys (LEN <= the workload's L, a multiple of 4; same B, H, d, N:M) next to the call on the "
                         "workload's padded arrays with the keys >= LEN masked; reported under extra")
    ap.add_argument("--products", choices=("fp32", "bf16x3"), default="bf16x3",
                    help="float workloads only: form the fp32 products on the fp32 matrix instruction (DFSS_F32) or "
                         "from bfloat16 pieces on the bf16 matrix pipe (DFSS_F32_BF16X3, the default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 64 MiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


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

    w = synth.WORKLOADS[args.workload]
    f32 = w.float32
    split = f32 and args.products == "bf16x3"
    s = Shape(w.B, w.H, w.L, w.L, w.d, w.N, w.M,
              (dfss.DFSS_F32_BF16X3 if split else dfss.DFSS_F32) if f32 else dfss.DFSS_BF16)
    if f32 and not split and (args.backward or args.key_padding or args.block_pattern):
        print("bench.py: with --products fp32 the float workloads run the plain forward pass only", file=sys.stderr)
        sys.exit(2)
    esz = 4 if f32 else 2
    # one-kernel paths exist for the 2-byte modes and, in the float mode, for bf16x3 products
    has_fused = (not f32) or split
    K, W = args.steps, args.warmup
    BH, L, d = w.BH, w.L, w.d

    # ---- buffers --------------------------------------------------------------------
    Qc, Kc, Vc = synth.make(w)
    ws_sparse = dfss.dfss_workspace_bytes(s)
    ws_dense = dfss.dense_workspace_bytes(s)
    set_bytes = 4 * BH * L * d * esz + max(ws_sparse, ws_dense)
    if args.warm:
        nsets = 1
    else:
        nsets = max(2, math.ceil(3 * LLC_BYTES / set_bytes))
    sets = []
    for i in range(nsets):
        sets.append(dict(
            Q=Qc.to(dev), K=Kc.to(dev), V=Vc.to(dev),
            O=torch.empty((BH, L, d), dtype=s.torch_dtype, device=dev),
            ws=torch.empty(max(ws_sparse, ws_dense), dtype=torch.uint8, device=dev)))
    torch.cuda.synchronize()

    # padded batch: additive key bias, 0 for real keys and -inf for padding (None = no mask)
    bias = None
    if args.key_padding:
        lengths = synth.padding_lengths(w.B, L, w.seed + 7)
        bias = synth.key_padding_bias(lengths, L).to(dev)

    block_mask, density = None, 1.0
    if args.block_pattern:
        bm = synth.block_pattern(L // 64, L // 64, seed=w.seed + 9, window=1, n_global=1, n_random=2)
        density = float(bm.float().mean())
        block_mask = bm.to(dev)

    def step_sparse(i):
        b = sets[i % nsets]
        if block_mask is not None:
            dfss.dfss_attention_blocked(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"])
        elif bias is None:
            dfss.dfss_attention(b["Q"], b["K"], b["V"], s, w.scale, O=b["O"], ws=b["ws"])
        else:
            dfss.dfss_attention_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"], ws=b["ws"])

    def step_dense(i):
        b = sets[i % nsets]
        if bias is None:
            dfss.dense_attention(b["Q"], b["K"], b["V"], s, w.scale, O=b["O"], ws=b["ws"])
        else:
            dfss.dense_attention_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"], ws=b["ws"])

    def step_dense_fused(i):
        b = sets[i % nsets]
        if block_mask is not None:
            dfss.dense_attention_fused_blocked(b["Q"], b["K"], b["V"], bias, block_mask, s, w.scale, O=b["O"])
        elif bias is None:
            dfss.dense_attention_fused(b["Q"], b["K"], b["V"], s, w.scale, O=b["O"])
        else:
            dfss.dense_attention_fused_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"])

    def step_sparse_staged(i):
        b = sets[i % nsets]
        dfss.dfss_attention_staged_bias(b["Q"], b["K"], b["V"], bias, s, w.scale, O=b["O"], ws=b["ws"])

    n_vals, n_meta = dfss.dfss_vals_bytes(s), dfss.dfss_meta_bytes(s)
    meta_at = (n_vals + 255) // 256 * 256

    def stage_buffers(b):
        """The kept values and the metadata inside the workspace, where dfss_attention puts them."""
        return b["ws"][:n_vals].view(s.torch_dtype), b["ws"][meta_at:meta_at + n_meta].view(torch.int16)

    def step_stage1(i):
        b = sets[i % nsets]
        vals, meta = stage_buffers(b)
        if bias is None:
            dfss.dfss_sddmm_prune(b["Q"], b["K"], s, w.scale, vals=vals, meta=meta)
        else:
            dfss.dfss_sddmm_prune_bias(b["Q"], b["K"], bias, s, w.scale, vals=vals, meta=meta)

    def step_stage2(i):
        b = sets[i % nsets]
        dfss.dfss_sparse_softmax(stage_buffers(b)[0], s)

    def step_stage3(i):
        b = sets[i % nsets]
        vals, meta = stage_buffers(b)
        dfss.dfss_spmm(vals, meta, b["V"], s, O=b["O"])

    def timed(step_fn, steps, warmup, use_graph=True):
        """Wall-clock of `steps` steps between two device synchronisations -> seconds."""
        for i in range(warmup):
            step_fn(i)
        torch.cuda.synchronize()
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(steps):
                    step_fn(i)
            g.replay()  # untimed: uploads the graph
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            g.replay()
            torch.cuda.synchronize()
            return time.perf_counter() - t0
        t0 = time.perf_counter()
        for i in range(steps):
            step_fn(i)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def event_avg_ms(step_fn, n):
        """Average launch duration of one kernel: n launches in one graph between two events
        recorded on the stream the kernels run on (the current PyTorch stream)."""
        for i in range(3):
            step_fn(i)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for i in range(n):
                step_fn(i)
        g.replay()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    if args.calibrate_copy:
        src = torch.ones(64 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    use_graph = not args.no_graph
    t_sparse = timed(step_sparse, K, W, use_graph)
    t_dense = timed(step_dense, K, W, use_graph)
    # the float mode has no fused kernels: dfss_attention already is the staged path there
    t_dense_fused = timed(step_dense_fused, K, W, use_graph) if has_fused else None
    t_staged = timed(step_sparse_staged, K, W, use_graph) if has_fused else t_sparse
    t_sparse_eager = timed(step_sparse, K, 0, False)

    # ---- per-kernel durations (events around a graph of K launches of one kernel) ------
    k_fused = event_avg_ms(step_sparse, K)       # dfss_attention is ONE kernel
    step_stage1(0)
    k1 = event_avg_ms(step_stage1, K)
    k2 = event_avg_ms(step_stage2, K)
    k3 = event_avg_ms(step_stage3, K)

    flops_alg = 3.0 * BH * L * L * d * density      # kept blocks only when a block pattern is given
    flops_eq = 4.0 * BH * L * L * d * density
    ms = t_sparse / K * 1e3
    ms_dense = t_dense / K * 1e3
    ms_dense_fused = t_dense_fused / K * 1e3 if has_fused else None
    ms_staged = t_staged / K * 1e3
    value = flops_alg / (t_sparse / K) / 1e12

    # Algorithmic work per launch.  Fused kernel: 3 L^2 d flops per head (2 L^2 d for Q K^T,
    # L^2 d for the half-dense P V), against the dense bf16 MFMA peak.  Stage kernels
    # (bytes per head): stage 1 reads Q,K = 4 L d and writes kept values L^2 plus metadata
    # L^2/8; stage 2 reads and writes L^2; stage 3 reads 1.125 L^2 + V and writes O.
    achieved = flops_alg / (k_fused * 1e-3) / 1e12
    # (float mode: every element is 4 bytes, the metadata again 1/16 of the dense matrix)
    bytes1 = BH * (2.0 * esz * L * d + (esz / 2 + esz / 16) * L * L)
    bytes2 = BH * (esz * L * L)
    bytes3 = BH * ((esz / 2 + esz / 16) * L * L + 2.0 * esz * L * d)
    flops1_stage = 2.0 * BH * L * L * d
    peak1 = MFMA_F32_PEAK_TFLOPS if f32 and not split else MFMA_BF16_PEAK_TFLOPS / (3.0 if f32 else 1.0)
    roof1 = min(peak1, HBM_PEAK_GBS * 1e9 * (flops1_stage / bytes1) / 1e12)
    kernels = {"sddmm_prune": (k1, bytes1), "sparse_softmax": (k2, bytes2), "spmm": (k3, bytes3)}

    out = {
        "metric": "DFSS attention forward TFLOP/s (algorithmic 3*BH*L^2*d per step)",
        "value": round(value, 3),
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
                   "key_padding": bool(args.key_padding),
                   "block_pattern": (f"window +-1, 1 global, 2 random blocks of 64 x 64, density {density:.3f}"
                                     if args.block_pattern else None), "buffer_sets": nsets, "cache": "warm" if args.warm else "cold (rotating buffer sets)",
                   "launch": "hip graph of all timed steps" if use_graph else "direct"},
        "roofline": {"bound": "mfma", "kernel": "k_fused (dfss_attention)", "achieved": round(achieved, 2),
                     "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get(w.name),
                     "algorithmic_hbm_bytes_per_launch": 8.0 * BH * L * d,
                     "avg_launch_ms": round(k_fused, 5), "algorithmic_flops_per_launch": flops_alg},
        "extra": {
            "speedup_vs_dense_attention_fused": round(ms_dense_fused / ms, 4) if has_fused else None,
            "speedup_vs_dense_attention_3stage": round(ms_dense / ms, 4),
            "staged_path_speedup_vs_dense_attention_3stage": round(ms_dense / ms_staged, 4),
            "dense_attention_fused_ms_per_step": round(ms_dense_fused, 5) if has_fused else None,
            "dense_attention_3stage_ms_per_step": round(ms_dense, 5),
            "dfss_attention_staged_ms_per_step": round(ms_staged, 5),
            "dense_equivalent_tflops": round(flops_eq / (t_sparse / K) / 1e12, 3),
            "dense_attention_fused_tflops": round(flops_eq / (t_dense_fused / K) / 1e12, 3) if has_fused else None,
            "ms_per_step_direct_launch": round(t_sparse_eager / K * 1e3, 5),
            "stage_kernel_ms": {k: round(v[0], 5) for k, v in kernels.items()},
            "stage_kernel_GBps": {k: round(v[1] / (v[0] * 1e-3) / 1e9, 1) for k, v in kernels.items()},
            "stage_kernel_frac_of_hbm_peak": {k: round(v[1] / (v[0] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
                                              for k, v in kernels.items()},
            "sddmm_prune_tflops": round(2.0 * BH * L * L * d / (k1 * 1e-3) / 1e12, 2),
            "sddmm_prune_frac_of_mfma_peak": round(flops1_stage / (k1 * 1e-3) / 1e12
                                                   / (MFMA_F32_PEAK_TFLOPS if f32 and not split
                                                      else MFMA_BF16_PEAK_TFLOPS), 4),
            # the lower of the two ceilings of stage 1: the matrix peak (a third of the bf16 peak where every
            # product is three bf16 products), or the HBM peak times the stage's flops per algorithmic byte
            # (Q, K read; kept values and metadata written)
            "sddmm_prune_roofline_tflops": round(roof1, 1),
            "sddmm_prune_frac_of_min_roofline": round(flops1_stage / (k1 * 1e-3) / 1e12 / roof1, 4),
        },
    }
    if f32:
        flops1 = 2.0 * BH * L * L * d
        ach1 = flops1 / (k1 * 1e-3) / 1e12
        if has_fused:
            # one kernel (k_fused_split) on the bf16 matrix pipe; every algorithmic product is executed as
            # three bf16 products, so a third of the bf16 peak is the most this route can reach
            out["roofline"]["kernel"] = "k_fused_split (dfss_attention, float data, bf16x3 products)"
            out["roofline"]["algorithmic_hbm_bytes_per_launch"] = 4.0 * esz * BH * L * d
            out["roofline"]["executed_matrix_flops_per_launch"] = 3.0 * flops_alg
        else:
            # three kernels per step; the score/prune kernel is the largest and is bound by the fp32 matrix
            # instruction: 2 L^2 d flops per head per launch
            out["roofline"] = {"bound": "mfma", "kernel": "k_scores_f32 (dfss_sddmm_prune, float data)",
                               "achieved": round(ach1, 2), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                               "frac": round(ach1 / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                               "algorithmic_hbm_bytes_per_launch": bytes1, "avg_launch_ms": round(k1, 5),
                               "algorithmic_flops_per_launch": flops1}
        out["extra"]["spmm_dense_equivalent_tflops"] = round(flops1 / (k3 * 1e-3) / 1e12, 2)

    if args.backward and block_mask is None:
        b = sets[0]
        vals = torch.empty((BH, L, s.Lc), dtype=s.torch_dtype, device=dev)
        meta = torch.empty((BH * L * s.meta_words,), dtype=torch.int16, device=dev)
        if bias is None:
            dfss.dfss_sddmm_prune(b["Q"], b["K"], s, w.scale, vals=vals, meta=meta)
        else:
            dfss.dfss_sddmm_prune_bias(b["Q"], b["K"], bias, s, w.scale, vals=vals, meta=meta)
        dfss.dfss_sparse_softmax(vals, s)
        O_fwd = dfss.dfss_spmm(vals, meta, b["V"], s)
        dO = torch.randn(BH, L, d, device=dev).to(s.torch_dtype)
        grads = [torch.empty((BH, L, d), dtype=s.torch_dtype, device=dev) for _ in range(3)]
        ws_b = torch.empty(dfss.dfss_backward_workspace_bytes(s), dtype=torch.uint8, device=dev)

        def step_backward(i):
            dfss.dfss_attention_backward(dO, b["Q"], b["K"], b["V"], O_fwd, vals, meta, s, w.scale,
                                         dQ=grads[0], dK=grads[1], dV=grads[2], ws=ws_b)

        t_bwd = timed(step_backward, K, W, use_graph)
        flops_bwd = 5.0 * BH * L * L * d      # dP: 2 L^2 d (formed densely), dQ, dK, dV: L^2 d each on kept entries
        out["extra"]["backward_ms_per_step"] = round(t_bwd / K * 1e3, 5)
        out["extra"]["backward_tflops"] = round(flops_bwd / (t_bwd / K) / 1e12, 2)
        out["extra"]["backward_over_staged_forward"] = round((t_bwd / K * 1e3) / ms_staged, 3)

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
        t_r = timed(lambda i: dfss.dfss_attention_ragged(Qr, Kr, Vr, None, sr, w.scale, O=Or), K, W, use_graph)
        t_rd = timed(lambda i: dfss.dense_attention_fused_ragged(Qr, Kr, Vr, None, sr, w.scale, O=Or), K, W, use_graph)
        t_p = timed(lambda i: dfss.dfss_attention_bias(b["Q"], b["K"], b["V"], pad_bias, s, w.scale, O=b["O"],
                                                       ws=b["ws"]), K, W, use_graph)
        out["extra"]["unpadded"] = {
            "length": Lr, "cache": "warm (one buffer set)",
            "dfss_attention_ragged_ms_per_step": round(t_r / K * 1e3, 5),
            "dense_attention_fused_ragged_ms_per_step": round(t_rd / K * 1e3, 5),
            "padded_and_masked_dfss_attention_bias_ms_per_step": round(t_p / K * 1e3, 5),
            "algorithmic_tflops": round(3.0 * BH * Lr * Lr * d / (t_r / K) / 1e12, 2)}

    if args.block_pattern:
        # only the fused kernels take a block pattern: the three-stage figures would be those of a
        # different function
        for k in ("speedup_vs_dense_attention_3stage", "staged_path_speedup_vs_dense_attention_3stage",
                  "dense_attention_3stage_ms_per_step", "dfss_attention_staged_ms_per_step", "stage_kernel_ms",
                  "stage_kernel_GBps", "stage_kernel_frac_of_hbm_peak", "sddmm_prune_tflops",
                  "sddmm_prune_frac_of_mfma_peak", "sddmm_prune_roofline_tflops",
                  "sddmm_prune_frac_of_min_roofline"):
            out["extra"][k] = None
        out["roofline"]["algorithmic_hbm_bytes_per_launch"] = None

    if not args.no_cpu_baseline:
        import oracle
        Qn, Kn, Vn = (synth.to_numpy_f32(t) for t in (Qc, Kc, Vc))
        # bounded sample: as many heads as fit in roughly 10-30 s of host work
        per_head_flops = 3.0 * L * L * d
        heads = int(max(1, min(BH, 2.0e10 // per_head_flops)))
        oracle.attention(Qn[:1], Kn[:1], Vn[:1], w.N, w.M, w.scale)  # load + warm
        reps, dt = 0, 0.0
        t0 = time.perf_counter()
        while dt < 10.0 and reps < 500:         # about ten seconds of host work, whole passes only
            oracle.attention(Qn[:heads], Kn[:heads], Vn[:heads], w.N, w.M, w.scale,
                             block_mask=None if block_mask is None else block_mask.cpu().numpy())
            reps += 1
            dt = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": round(reps * heads * per_head_flops / dt / 1e12, 6), "unit": "TFLOP/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{heads} of {BH} heads of {w.name}, {reps} passes in {dt:.2f} s"}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
