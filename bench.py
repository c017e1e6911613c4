#!/usr/bin/env python3
"""Benchmark of the subsampled-global-attention hot path on one MI355X.

One "step" = one layer's pass of the whole path on resident inputs:
``agg_kv_subsample`` (index list, grid gather, mean terms) followed by
``agg_global_attn_fwd``.  The dense s = 1 baseline (``agg_dense_global_attn_fwd``)
is timed beside it, not inside the step.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload f100|f300|f333|f800|tiny]
                  [--also f300,f800] [--no-dense] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "ms/layer & TFLOP/s (frac of bf16 peak) for subsampled global attn, 100/300/800 frames"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak (256 CU x 4 SIMD x 1024 flop/clk x 2.4 GHz)
PEAK_HBM_GBS = 8000.0


def sga_flops(NQ, M, H, D):
    # QK^T and PV, 2 flops per multiply-add, all heads; +2 columns for the self and mean terms
    return 4.0 * NQ * (M + 2) * D * H


def time_events(fn, steps, warmup):
    """Average milliseconds of fn() over `steps` launches, HIP events on torch's current
    stream (the stream every library call here is enqueued on)."""
    import torch

    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    start = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    stop = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    for i in range(steps):
        start[i].record()
        fn()
        stop[i].record()
    torch.cuda.synchronize()
    ms = [a.elapsed_time(b) for a, b in zip(start, stop)]
    return sum(ms) / len(ms), min(ms)


def run_workload(name, steps, warmup, dense, log):
    import torch

    from paper_2512_02541_amd import binding as agg
    from paper_2512_02541_amd import harness, inputs

    w = inputs.WORKLOADS[name]
    shape = harness.shape_of(w)
    log("generating %s (%d frames, %d tokens)" % (name, w.N, w.NQ))
    q, k, v = inputs.make_qkv(w, "cuda")
    buf = harness.alloc(shape, "cuda")
    torch.cuda.synchronize()

    def step():
        harness.subsample(buf, k, v)
        harness.attend(buf, q, k, v)

    # whole step: wall clock bracketed by synchronize, exactly `steps` passes
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / steps

    ms_gather, _ = time_events(lambda: harness.subsample(buf, k, v), steps, 1)
    ms_attn, ms_attn_min = time_events(lambda: harness.attend(buf, q, k, v), steps, 1)

    flops = sga_flops(w.NQ, buf.M, w.H, w.D)
    C = w.H * w.D
    gather_bytes = 2.0 * w.NQ * C * 2 + 2.0 * buf.M * C * 2  # K,V read once; kept rows written once
    res = {
        "workload": name, "frames": w.N, "NQ": w.NQ, "M": buf.M, "n_dropped": buf.n_dropped,
        "strides": [w.s_h, w.s_w],
        "ms_layer": ms_step, "ms_gather": ms_gather, "ms_attn": ms_attn, "ms_attn_min": ms_attn_min,
        "tflops_layer": flops / (ms_step * 1e-3) / 1e12,
        "tflops_attn": flops / (ms_attn * 1e-3) / 1e12,
        "frac_peak_attn": flops / (ms_attn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "gather_gbs": gather_bytes / (ms_gather * 1e-3) / 1e9,
        "gather_frac_hbm": gather_bytes / (ms_gather * 1e-3) / 1e9 / PEAK_HBM_GBS,
        "flops_per_layer": flops, "gather_bytes": gather_bytes,
    }
    # the same layer with the kernel reading the kept rows in place through the index list
    Oi = torch.empty_like(buf.O)
    ms_idx, _ = time_events(lambda: agg.agg_global_attn_fwd_idx(
        shape, q, k, v, buf.idx, buf.kmean, buf.vmean, Oi, None), max(2, min(steps, 3)), 1)
    res.update({"ms_attn_idx": ms_idx, "tflops_attn_idx": flops / (ms_idx * 1e-3) / 1e12})
    del Oi
    if dense:
        # what a fallback costs: one query in 256 gets logits far outside the fast path's window,
        # so EVERY workgroup redoes its rows in the general path (second kernel of the call)
        qx = q.clone()
        qx[:, ::256] *= 64.0
        Ox = buf.O
        buf.O = torch.empty_like(Ox)
        ms_fb, _ = time_events(lambda: harness.attend(buf, qx, k, v), max(2, min(steps, 3)), 1)
        buf.O = Ox
        del qx
        res["general_path"] = {
            "what": "attention launch with every workgroup falling back to the general path "
                    "(one query in 256 scaled by 64)",
            "ms_attn_all_fallback": ms_fb, "ms_attn_fast": ms_attn,
            "ratio": ms_fb / ms_attn, "tflops_all_fallback": flops / (ms_fb * 1e-3) / 1e12}
        # a plain device copy of 1 GiB: the HBM rate this part reaches (read + write bytes)
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        ms_copy, _ = time_events(lambda: dst.copy_(src), 5, 2)
        res["copy_gbs"] = 2.0 * src.numel() * 4 / (ms_copy * 1e-3) / 1e9
        del src, dst
        Od = torch.empty_like(buf.O)

        def dense_step():
            agg.agg_dense_global_attn_fwd(shape, q, k, v, Od, None)

        ms_dense, _ = time_events(dense_step, max(1, min(steps, 3)), 1)
        dflops = 4.0 * w.NQ * w.NQ * w.D * w.H
        res.update({"ms_dense": ms_dense, "tflops_dense": dflops / (ms_dense * 1e-3) / 1e12,
                    "speedup_vs_dense": ms_dense / ms_step,
                    "ideal_speedup": w.NQ / buf.M})
        # frame attention (Global-to-Frame conversion of an early global block), same tensors
        ms_frame, _ = time_events(
            lambda: agg.agg_frame_attn_fwd(shape, q, k, v, Od, None), max(1, min(steps, 3)), 1)
        fflops = 4.0 * w.N * w.L * w.L * w.D * w.H
        res.update({"ms_frame_attn": ms_frame, "tflops_frame_attn": fflops / (ms_frame * 1e-3) / 1e12})
        del Od
    return res, (w, shape, q, k, v, buf)


def cpu_baseline(w, shape, q, k, v, buf, flops, nrows, log):
    """The oracle, as it stands, on the host's cores: gather + mean in full, attention on
    `nrows` evenly spaced query rows; also used to re-check the GPU output."""
    import numpy as np

    from oracle import sga_oracle as orc
    from paper_2512_02541_amd import inputs

    o = orc.Shape(shape.B, shape.N, shape.n_h, shape.n_w, shape.n_special, shape.H, shape.D,
                  shape.s_h, shape.s_w, shape.keep_first_frame, shape.flags, shape.scale,
                  shape.mean_logit_bias)
    qb, kb, vb = (inputs.bf16_bits(t) for t in (q, k, v))
    log("oracle: gather + mean in full")
    t0 = time.perf_counter()
    idx = orc.kept_indices(o)
    M, nd = orc.counts(o)
    Kc, Vc = orc.gather(o, kb, vb, idx)
    km, vm = orc.mean(o, kb, vb)
    t_pre = time.perf_counter() - t0
    rows = np.unique(np.linspace(0, shape.NQ - 1, nrows).astype(np.int64))
    log("oracle: attention on %d sampled rows" % len(rows))
    t0 = time.perf_counter()
    want, _, _ = orc.attn_rows(o, qb, kb, vb, Kc, Vc, km, vm, nd, rows)
    t_rows = time.perf_counter() - t0
    t_full = t_pre + t_rows * shape.NQ / len(rows)
    got = buf.O[:, rows].float().cpu().numpy().astype(np.float64)
    err = np.abs(got - want)
    base = {
        "value": flops / t_full / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(),
        "kind": "oracle",
        "sample": "gather+mean in full (%.2f s); attention on %d of %d query rows x %d heads "
                  "against the full compacted set (%.2f s), extrapolated linearly to all rows "
                  "(%.0f s per layer)" % (t_pre, len(rows), shape.NQ, shape.H, t_rows, t_full),
        "rows_per_s": len(rows) / t_rows, "extrapolated_s_per_layer": t_full,
    }
    parity = {"rows": int(len(rows)), "max_abs": float(err.max()), "mean_abs": float(err.mean())}
    return base, parity


def read_traffic(name):
    """HBM bytes per attention launch from the committed rocprofv3 counter summary, if any."""
    path = os.path.join(ROOT, "profiles", "sga_attn_%s_pmc.txt" % name)
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def run_only(args, log):
    """Launches one piece of the path `steps` times, nothing else: short runs for
    rocprofv3 counter collection.  `copy` is a plain device copy of 1 GiB whose known
    size calibrates the FETCH_SIZE / WRITE_SIZE counters."""
    import torch

    from paper_2512_02541_amd import binding as agg
    from paper_2512_02541_amd import harness, inputs

    if args.only == "copy":
        src = torch.zeros(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        ms, mn = time_events(lambda: dst.copy_(src), args.steps, 1)
        print(json.dumps({"only": "copy", "bytes_read": src.numel() * 4,
                          "bytes_written": src.numel() * 4, "launches": args.steps + 1,
                          "ms": ms, "gbs_read_plus_write": 2 * src.numel() * 4 / (ms * 1e-3) / 1e9}))
        return 0
    w = inputs.WORKLOADS[args.workload]
    shape = harness.shape_of(w)
    log("generating %s (%s)" % (args.workload, args.data))
    if args.data == "zeros":      # same launches on all-zero tensors: isolates the effect of the
        q = k = v = torch.zeros((w.B, w.NQ, w.H, w.D), dtype=torch.bfloat16, device="cuda")  # chip's power management
    elif args.data == "iid":
        q, k, v = inputs.iid_qkv(w.B, w.NQ, w.H, w.D, w.seed, "cuda")
    else:
        q, k, v = inputs.make_qkv(w, "cuda")
        if args.data == "extreme":  # one query in 256 with logits far outside the fast path's
            q[:, ::256] *= 64.0     # window: every workgroup falls back to the general path
    buf = harness.alloc(shape, "cuda")
    harness.subsample(buf, k, v)
    torch.cuda.synchronize()
    log("inputs ready; launching %s x %d" % (args.only, args.steps))
    if args.only == "attn" and args.steps >= 5:
        ms, mn = time_events(lambda: harness.attend(buf, q, k, v), args.steps, 2)
        fl = sga_flops(w.NQ, buf.M, w.H, w.D)
        print(json.dumps({"only": "attn", "workload": args.workload, "data": args.data,
                          "launches": args.steps + 2, "ms_attn": ms, "ms_attn_min": mn,
                          "tflops_attn": fl / (ms * 1e-3) / 1e12,
                          "frac_peak": fl / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}))
        return 0
    if args.only == "gather" and args.steps >= 5:
        ms, mn = time_events(lambda: harness.subsample(buf, k, v), args.steps, 2)
        nbytes = 2.0 * w.NQ * w.H * w.D * 2 + 2.0 * buf.M * w.H * w.D * 2
        print(json.dumps({"only": "gather", "workload": args.workload, "launches": args.steps + 2,
                          "ms_gather": ms, "ms_gather_min": mn,
                          "gather_gbs": nbytes / (ms * 1e-3) / 1e9}))
        return 0
    for i in range(args.steps):
        if args.only == "attn":
            harness.attend(buf, q, k, v)
        elif args.only == "gather":
            harness.subsample(buf, k, v)
        else:
            agg.agg_dense_global_attn_fwd(shape, q, k, v, buf.O, None)
        torch.cuda.synchronize()
        log("launch %d done" % i)
    print(json.dumps({"only": args.only, "workload": args.workload, "launches": args.steps,
                      "flops_per_launch": sga_flops(w.NQ, buf.M, w.H, w.D),
                      "gather_bytes": 2.0 * w.NQ * w.H * w.D * 2 + 2.0 * buf.M * w.H * w.D * 2}))
    return 0


def run_sweep(args, log):
    """Variant sweep of Sec. 4.3 and its ablations on one workload's tensors: every sigma of the
    paper's table, VGGT (first frame kept) and pi^3 (all frames subsampled) rules, and the
    SubsampleOnly / WithDiagonal / WithMean / both flag combinations."""
    import torch

    from paper_2512_02541_amd import binding as agg
    from paper_2512_02541_amd import harness, inputs

    w = inputs.WORKLOADS[args.workload]
    q, k, v = inputs.make_qkv(w, "cuda")
    rows = []
    cases = [(sig, 1, 3) for sig in (2, 4, 6, 9)] + [(sig, 0, 3) for sig in (2, 4, 6, 9)] + \
            [(w.s_h * w.s_w, 1, fl) for fl in (0, 1, 2)]
    for sigma, keep_first, flags in cases:
        s_h, s_w = agg.agg_sigma_to_strides(sigma)
        shape = harness.shape_of(w, flags=flags, s_h=s_h, s_w=s_w, keep_first_frame=keep_first)
        buf = harness.alloc(shape, "cuda", with_lse=False)
        ms_g, _ = time_events(lambda: harness.subsample(buf, k, v), args.steps, 1)
        ms_a, _ = time_events(lambda: harness.attend(buf, q, k, v), args.steps, 1)
        fl_ = sga_flops(w.NQ, buf.M, w.H, w.D)
        rows.append({"sigma": sigma, "keep_first_frame": keep_first, "flags": flags, "M": buf.M,
                     "ms_gather": ms_g, "ms_attn": ms_a, "tflops_attn": fl_ / (ms_a * 1e-3) / 1e12})
        log("sigma %d keep_first %d flags %d: M %d gather %.3f ms attn %.2f ms" % (
            sigma, keep_first, flags, buf.M, ms_g, ms_a))
        del buf
        torch.cuda.empty_cache()
    # token-selection ablation (supplementary material): one token per window chosen at random
    # or by feature magnitude, run through the list-driven entry points
    shape = harness.shape_of(w)
    M, _ = agg.agg_kv_count(shape)
    list_rows = []
    for rule, name in ((agg.AGG_SELECT_FIRST, "first"), (agg.AGG_SELECT_RANDOM, "random"),
                       (agg.AGG_SELECT_HIGH, "high"), (agg.AGG_SELECT_LOW, "low")):
        lst = torch.empty((w.B, M), dtype=torch.int32, device="cuda")
        ms_sel, _ = time_events(lambda: agg.agg_select_kv_indices(shape, rule, 7, k, lst), args.steps, 1)
        lb = harness.list_forward(shape, lst, q, k, v)
        ms_sub, _ = time_events(lambda: agg.agg_kv_subsample_list(
            shape, lst, M, k, v, lb.Kc, lb.Vc, lb.kmean, lb.vmean, lb.kept_bits, lb.n_dropped,
            lb.workspace, lb.workspace.numel()), args.steps, 1)
        ms_att, _ = time_events(lambda: agg.agg_global_attn_fwd_list(
            shape, M, q, k, v, lb.Kc, lb.Vc, lb.kmean, lb.vmean, lb.kept_bits, lb.n_dropped, lb.O,
            None), args.steps, 1)
        list_rows.append({"rule": name, "M": M, "ms_select": ms_sel, "ms_subsample_list": ms_sub,
                          "ms_attn_list": ms_att})
        log("rule %s: select %.3f ms, list gather+mean %.3f ms, attn %.2f ms" % (
            name, ms_sel, ms_sub, ms_att))
        del lb, lst
        torch.cuda.empty_cache()
    # cell-mean variant: pooled compacted set, attention without extras
    pb = harness.pool_forward(shape, q, k, v)
    ms_pool, _ = time_events(lambda: agg.agg_kv_pool(pb.shape, k, v, pb.Kc, pb.Vc), args.steps, 1)
    ms_patt, _ = time_events(lambda: harness.attend(pb, q, k, v), args.steps, 1)
    list_rows.append({"rule": "cell_mean", "M": M, "ms_select": 0.0, "ms_subsample_list": ms_pool,
                      "ms_attn_list": ms_patt})
    log("rule cell_mean: pooling %.3f ms, attn %.2f ms" % (ms_pool, ms_patt))
    print(json.dumps({"sweep": args.workload, "NQ": w.NQ, "rows": rows, "selection_rules": list_rows}))
    return 0


def time_block_stack(workload, layers_n, t_early, t_end, steps, warmup, with_dense, log):
    """Times the chained global-attention blocks on `workload` (see run_block) and returns a
    dict: ms per pass over the stack, one block of each kind alone, and the attention and gather
    launches of a subsampled block alone (what remains is LayerNorm + projections)."""
    import torch

    from paper_2512_02541_amd import binding as agg
    from paper_2512_02541_amd import harness, inputs

    w = inputs.WORKLOADS[workload]
    shape = harness.shape_of(w)
    C = w.H * w.D
    log("block stack on %s: %d tokens x %d channels, %d layers (%d as frame attention)" % (
        workload, w.NQ, C, layers_n, t_early))
    x0 = inputs.block_input(w.B, w.NQ, C, w.seed, "cuda")
    layers = [inputs.block_weights(C, w.seed + 1 + i, "cuda") for i in range(layers_n)]
    cws = [agg.make_block_weights(l["ln_gamma"], l["ln_beta"], l["ln_eps"], l["w_q"], l["w_k"],
                                  l["w_v"], l["w_o"], l["b_q"], l["b_k"], l["b_v"], l["b_o"])
           for l in layers]
    t_end = layers_n - 1 if t_end is None else t_end
    modes = [agg.AGG_BLOCK_FRAME if (i < t_early or i > t_end) else agg.AGG_BLOCK_SGA
             for i in range(layers_n)]
    n_frame = sum(m == agg.AGG_BLOCK_FRAME for m in modes)
    nws = max(agg.agg_block_workspace_bytes(shape, m) for m in
              (agg.AGG_BLOCK_FRAME, agg.AGG_BLOCK_SGA, agg.AGG_BLOCK_DENSE))
    ws = torch.empty(nws, dtype=torch.uint8, device="cuda")
    xa, xb = torch.empty_like(x0), torch.empty_like(x0)

    def stack():
        src = x0
        for i in range(layers_n):
            dst = xa if (i % 2 == 0) else xb
            agg.agg_global_block_fwd(shape, modes[i], cws[i], src, dst, ws, nws)
            src = dst
        return src

    for _ in range(warmup):
        stack()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        out = stack()
    torch.cuda.synchronize()
    ms_stack = (time.perf_counter() - t0) * 1e3 / steps
    finite = bool(torch.isfinite(out[:, ::997].float()).all().item())

    def one(mode, n):
        return time_events(lambda: agg.agg_global_block_fwd(shape, mode, cws[-1], x0, xa, ws, nws),
                           n, 1)[0]

    ms_sga = one(agg.AGG_BLOCK_SGA, steps)
    ms_frame = one(agg.AGG_BLOCK_FRAME, steps)
    ms_dense = one(agg.AGG_BLOCK_DENSE, 1) if with_dense else None
    # the attention-side launches of one block alone, on the block's own Q/K/V (left in the
    # workspace by the last call: five [B, NQ, C] activations, then the attention scratch)
    act = (w.B * w.NQ * C * 2 + 255) // 256 * 256
    qv, kv, vv = (ws[i * act:i * act + w.B * w.NQ * C * 2].view(torch.bfloat16).view(
        w.B, w.NQ, w.H, w.D) for i in (1, 2, 3))
    buf = harness.alloc(shape, "cuda", with_lse=False)
    ms_gather = time_events(lambda: harness.subsample(buf, kv, vv), steps, 1)[0]
    ms_attn = time_events(lambda: harness.attend(buf, qv, kv, vv), steps, 1)[0]
    ms_fattn = time_events(lambda: agg.agg_frame_attn_fwd(shape, qv, kv, vv, buf.O, None), steps, 1)[0]
    M, _ = agg.agg_kv_count(shape)
    proj_flops = 4 * 2.0 * w.NQ * C * C
    fl_attn = sga_flops(w.NQ, M, w.H, w.D)
    fl_sga = fl_attn + proj_flops
    fl_frame = 4.0 * w.N * w.L * w.L * w.D * w.H + proj_flops
    fl_stack = n_frame * fl_frame + (layers_n - n_frame) * fl_sga
    return {
        "workload": "%s block stack: %d frames x (37x37+5) tokens, dim %d, %d global blocks, first "
                    "%d%s as frame attention, rest subsampled with strides (%d,%d), diag+mean" % (
                        workload, w.N, C, layers_n, t_early,
                        "" if t_end == layers_n - 1 else " and those above index %d" % t_end,
                        w.s_h, w.s_w),
        "NQ": w.NQ, "M": M, "passes_timed": steps, "ms_stack": ms_stack,
        "ms_block_sga": ms_sga, "ms_block_frame": ms_frame, "ms_block_dense": ms_dense,
        "ms_sga_attention_kernel": ms_attn, "ms_sga_gather": ms_gather,
        "ms_frame_attention_kernel": ms_fattn,
        "ms_layernorm_and_projections": ms_sga - ms_attn - ms_gather,
        "frac_peak_sga_attention": fl_attn / (ms_attn * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "tflops_block_sga": fl_sga / (ms_sga * 1e-3) / 1e12,
        "tflops_block_frame": fl_frame / (ms_frame * 1e-3) / 1e12,
        "tflops_stack": fl_stack / (ms_stack * 1e-3) / 1e12,
        "projection_flops_per_block": proj_flops,
        "ms_stack_if_all_dense": (ms_dense * layers_n) if ms_dense else None,
        "speedup_vs_all_dense": (ms_dense * layers_n / ms_stack) if ms_dense else None,
        "output_finite": finite,
    }


def run_block(args, log):
    """The global-attention blocks of one aggregator pass at full width (dim 1024 = 16 x 64):
    LayerNorm, Q/K/V projections, attention, output projection and residual per block;
    `--layers` blocks chained, the first `--t-early` of them as per-frame attention
    (Global-to-Frame conversion, Sec. 4.2), the rest subsampled (Sec. 4.3).  One dense
    block is timed beside them for the ratio.  Random-init weights, one set per layer."""
    r = time_block_stack(args.workload, args.layers, args.t_early, args.t_end, args.steps,
                         args.warmup, not args.no_dense, log)
    res = {
        "metric": "ms per aggregator pass over the global-attention blocks (LayerNorm + QKV "
                  "projection + attention + output projection + residual)",
        "value": r["ms_stack"], "unit": "ms", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_stack"], "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic", "config": r,
    }
    print(json.dumps(res), flush=True)
    return 0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="f100")
    ap.add_argument("--also", default="f300,f800",
                    help="comma list of further workloads timed (SGA only) into config.also")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-block", action="store_true",
                    help="skip the 12-block stack at 333 frames (config.block_f333)")
    ap.add_argument("--cpu-rows", type=int, default=1024)
    ap.add_argument("--sweep", action="store_true",
                    help="time the method's variants on --workload (sigma 2/4/6/9, both first-frame "
                         "rules, the four diag/mean flag combinations) and print one JSON line")
    ap.add_argument("--block", action="store_true",
                    help="time the chained global-attention blocks (LayerNorm, projections, "
                         "attention, residual) on --workload instead of the bare attention path")
    ap.add_argument("--layers", type=int, default=12)
    ap.add_argument("--t-end", type=int, default=None,
                    help="with --block: blocks with index above this also run as per-frame attention "
                         "(the paper's ablation on the last global layers); default: none")
    ap.add_argument("--t-early", type=int, default=4,
                    help="with --block: leading blocks run as per-frame attention")
    ap.add_argument("--data", choices=["structured", "iid", "zeros", "extreme"], default="structured",
                    help="with --only: values of Q/K/V (zeros shows what the same instruction stream "
                         "reaches when the operands do not toggle)")
    ap.add_argument("--only", choices=["attn", "gather", "dense", "copy"], default=None,
                    help="profiling aid: launch just this piece `steps` times (for rocprofv3 runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        return 2

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    from paper_2512_02541_amd import binding as agg

    agg.lib()  # fail loudly if the HIP library is missing

    if args.only:
        return run_only(args, log)
    if args.sweep:
        return run_sweep(args, log)
    if args.block:
        return run_block(args, log)

    res, ctx = run_workload(args.workload, args.steps, args.warmup, not args.no_dense, log)
    cpu, parity = (None, None)
    if not args.no_cpu:
        cpu, parity = cpu_baseline(*ctx, res["flops_per_layer"], args.cpu_rows, log)
    del ctx
    torch.cuda.empty_cache()

    also = []
    for name in [x for x in args.also.split(",") if x and x != args.workload]:
        r, c = run_workload(name, max(2, args.steps // 3), 1, False, log)
        del c
        torch.cuda.empty_cache()
        also.append({k: r[k] for k in ("workload", "frames", "NQ", "M", "strides", "ms_layer",
                                       "ms_gather", "ms_attn", "tflops_attn", "frac_peak_attn",
                                       "gather_gbs", "ms_attn_idx")})

    block = None
    if not args.no_block:
        # BASELINE config 5: 12 global blocks at 333 frames, the first 4 as frame attention
        block = time_block_stack("f333", 12, 4, None, 2, 1, False, log)
        torch.cuda.empty_cache()

    out = {
        "metric": METRIC,
        "value": res["tflops_layer"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": res["ms_layer"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d frames x (37x37+5) tokens, 16 heads x 64, strides (%d,%d), "
                               "diag+mean, first frame kept" % (res["workload"], res["frames"],
                                                                res["strides"][0], res["strides"][1])
                   if res["workload"] != "tiny" else "tiny",
                   "NQ": res["NQ"], "M": res["M"], "n_dropped": res["n_dropped"],
                   "ms_gather": res["ms_gather"], "ms_attn": res["ms_attn"],
                   "gather_gbs": res["gather_gbs"], "gather_frac_hbm": res["gather_frac_hbm"],
                   "copy_gbs": res.get("copy_gbs"), "general_path": res.get("general_path"),
                   "frac_bf16_peak_layer": res["tflops_layer"] / PEAK_BF16_TFLOPS,
                   "ms_dense": res.get("ms_dense"), "tflops_dense": res.get("tflops_dense"),
                   "ms_frame_attn": res.get("ms_frame_attn"),
                   "tflops_frame_attn": res.get("tflops_frame_attn"),
                   "ms_attn_idx": res.get("ms_attn_idx"),
                   "tflops_attn_idx": res.get("tflops_attn_idx"),
                   "speedup_vs_dense": res.get("speedup_vs_dense"),
                   "ideal_speedup": res.get("ideal_speedup"),
                   "paper_context": "end-to-end speedups ~2x/4-5x/8-10x at 100/300/800 frames on "
                                    "A100-80GB with FlashAttention-2 (whole model, not this layer)",
                   "also": also, "block_f333": block, "parity_vs_oracle": parity},
        "roofline": {"bound": "mfma", "achieved": res["tflops_attn"], "peak": PEAK_BF16_TFLOPS,
                     "unit": "TFLOP/s", "frac": res["frac_peak_attn"],
                     "traffic": read_traffic(res["workload"]),
                     "kernel": "sga_attn_kernel", "ms": res["ms_attn"]},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
