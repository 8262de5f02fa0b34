#!/usr/bin/env python3
"""Benchmark of the DaSS hot path on one MI355X.

One "step" is one pass of the whole hot path over one synthetic calibration
batch, inputs resident in HBM:
  stage 1  dass_calib_norms over all calibration tokens (chunked if the config
           says so), giving the f32 activation norms;
  stage 2  dass_score_mask_nm_batched on fresh copies of the block's Gate, Up (alpha
           0.5, groups down the rows) and Down (alpha 1, groups along the rows), pruned
           in place: Gate and Up share one launch, Down is a second one.

Prints ONE JSON line.  `value` is calibration tokens per second of the whole
step.  `roofline` is for the dominant kernel (the stage-1 MFMA kernel, > 99 % of
the step); `roofline_stage2` is the N:M launches (two) of the same timed steps,
bracketed by HIP events on the launch stream (stage 1 has just streamed 2 GB
through the caches, so the weights come from HBM).  `stage2.cold_*` repeats one
launch at a time on copies that rotate through more memory than the 256 MB
last-level cache.  `cpu_baseline` times the float64 oracle on this machine's
host cores on a bounded sample.

Beside the headline the same line carries the rest of the report: `roofline_stage2_48` (the
workload's matrices at 4:8, in a step and launch by launch), `stage2_other_reading` (Gate-Proj
with the groups along the input dimension), `unstructured` (50 % per comparison group, per
matrix), and `all_configs` (stage 1 and stage 2 of every other configuration, a few steps each).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM/fabric bytes per launch from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` runs of this
# benchmark (default workload), each scaled by what the counter reads for a plain copy of known
# size (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0; see profiles/).  A figure only stands while the source
# of its kernel is the one the counters were taken on; otherwise `traffic` is null.
MEASURED_TRAFFIC = {
    "stage1": {"sources": ("calib.hip",), "sha256": "32f3e49d551e12f84e1d9c3a627c4ffdcb1d80bd535600bb278f4661e9586e2c",
               "bytes": (42365400 * 2.0 + 88064) * 1024},
    # the step's two batched launches: Gate + Up, Down
    "stage2": {"sources": ("nm.hip", "select.h"), "sha256": "59a2ddf16cfc324fc9097880e39ca2c036a6a5ac0261dfce7b7d1d9f3f26e98c",
               "bytes": ((88443.7 * 2.0 + 176132.0) + (44497.5 * 2.0 + 88070.8)) * 1024},
}


def measured_traffic(which: str, is_default_workload: bool):
    import hashlib
    rec = MEASURED_TRAFFIC[which]
    h = hashlib.sha256()
    for name in rec["sources"]:
        with open(os.path.join(ROOT, "paper_2405_01943_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return rec["bytes"] if is_default_workload and h.hexdigest() == rec["sha256"] else None


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", default="llama2_7b")
    ap.add_argument("--tokens", type=int, default=0, help="override the token count (debugging)")
    ap.add_argument("--nm", default="2:4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--model-layers", type=int, default=32,
                    help="layers of the whole-model stage-2 measurement (0 skips it)")
    ap.add_argument("--stage2-launches", type=int, default=24)
    ap.add_argument("--other-configs", default="all",
                    help="'all', 'none' or a comma-separated list: configurations reported under all_configs")
    ap.add_argument("--other-steps", type=int, default=3)
    return ap.parse_args()


def make_inputs(cfg, dev):
    """X, Wgate, Wup, Wdown of a configuration, generated on the device chunk by chunk."""
    import torch

    from paper_2405_01943_amd import synth

    T = cfg.tokens
    gen_chunk = min(T, 32768)
    X = torch.empty((T, cfg.d), dtype=cfg.torch_dtype, device=dev)
    for c in range((T + gen_chunk - 1) // gen_chunk):
        lo = c * gen_chunk
        n = min(gen_chunk, T - lo)
        X[lo:lo + n] = synth.make_x(cfg, c, n, dev)
    Wg, Wu, Wd = (synth.make_weight(cfg, w, dev) for w in ("wg", "wu", "wd"))
    return X, Wg, Wu, Wd


def run_steps(cfg, n_keep, m, X, Wg, Wu, Wd, steps, warmup):
    """`warmup` untimed and `steps` timed passes of the hot path (calibration norms over all tokens,
    then the three N:M masks on fresh copies).  Returns (wall ms per step, stage-1 ms, stage-2 ms, norms);
    the stage times are means of HIP-event intervals on the launch stream."""
    import torch

    import paper_2405_01943_amd as dass

    dev = X.device
    T, d, I = cfg.tokens, cfg.d, cfg.d_int
    sumsq = torch.empty(I, device=dev)
    norms = torch.empty(I, device=dev)
    # stage 2 works in place: every step prunes its own fresh copies of the three matrices, all of them
    # resident before the timed region starts
    fresh = [tuple(w.clone() for w in (Wg, Wu, Wd)) for _ in range(warmup + steps)]
    task_sets = [[(g, norms, "rows", "rows", cfg.alpha_gate_up), (u, norms, "rows", "rows", cfg.alpha_gate_up),
                  (dn, norms, "cols", "cols", cfg.alpha_down)] for g, u, dn in fresh]
    ws_nm = torch.empty(max(16, dass.nm_batched_workspace_bytes(task_sets[0])), dtype=torch.uint8, device=dev)
    chunks = [(lo, min(cfg.chunk, T - lo)) for lo in range(0, T, cfg.chunk)]
    ev = lambda: torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    todo = iter(task_sets)

    def step():
        tasks = next(todo)
        e = [ev() for _ in range(3)]
        e[0].record()
        for k, (lo, n) in enumerate(chunks):
            dass.calib_norms(X[lo:lo + n], Wg, Wu, cfg.act, sumsq, accumulate=k > 0,
                             norms_out=norms if k == len(chunks) - 1 else None)
        e[1].record()
        # one call for the block's three matrices: Gate and Up (one shape) share a launch, Down follows
        dass.score_mask_nm_batched(tasks, n_keep, m, workspace=ws_nm)
        e[2].record()
        return e

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    evs = [step() for _ in range(steps)]
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    s1 = sum(e[0].elapsed_time(e[1]) for e in evs) / steps
    s2 = sum(e[1].elapsed_time(e[2]) for e in evs) / steps
    return wall * 1e3 / steps, s1, s2, norms


def cold_launch_us(W0, launch, n_launches, n_copies):
    """One launch at a time on copies of W0 that rotate through more memory than the 256 MB
    last-level cache; every copy is restored and the others are touched before it is timed.
    `launch(w)` enqueues the call under test on w.  Returns median and minimum in microseconds."""
    import torch

    ev = lambda: torch.cuda.Event(enable_timing=True)
    copies = [W0.clone() for _ in range(n_copies)]
    times = []
    for it in range(n_launches + 4):
        w = copies[it % n_copies]
        w.copy_(W0)
        for other in copies:
            if other is not w:
                other.add_(0)
        a, b = ev(), ev()
        a.record()
        launch(w)
        b.record()
        torch.cuda.synchronize()
        if it >= 4:
            times.append(a.elapsed_time(b))
    del copies
    return {"median_us": statistics.median(times) * 1e3, "min_us": min(times) * 1e3}


def cpu_baseline(cfg, n_keep, m, Wg, Wu, Wd, X_sample, norms32):
    """Time the oracle as it stands: stage 1 on a token slice x all neurons, stage 2 on the three
    full matrices; scale stage 1 linearly to the config's token count."""
    import numpy as np
    import torch

    import oracle

    f32 = lambda t: t.cpu().to(torch.float32).numpy()
    xs, wg, wu, wd = f32(X_sample), f32(Wg), f32(Wu), f32(Wd)
    t0 = time.perf_counter()
    oracle.sumsq(xs, wg, wu, cfg.act)
    t1 = time.perf_counter() - t0
    s1_rate = xs.shape[0] / t1
    t0 = time.perf_counter()
    oracle.mask_nm(wg, norms32, "rows", "rows", cfg.alpha_gate_up, n_keep, m)
    oracle.mask_nm(wu, norms32, "rows", "rows", cfg.alpha_gate_up, n_keep, m)
    oracle.mask_nm(wd, norms32, "cols", "cols", cfg.alpha_down, n_keep, m)
    t2 = time.perf_counter() - t0
    step_s = cfg.tokens / s1_rate + t2
    return {
        "value": cfg.tokens / step_s, "unit": "tokens/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": (f"stage 1: all {cfg.d_int} neurons x first {xs.shape[0]} tokens in {t1:.1f} s "
                   f"(scaled linearly to {cfg.tokens} tokens); stage 2: the three full matrices "
                   f"in {t2:.2f} s"),
        "stage1_tokens_per_s": s1_rate,
        "stage2_GBps": 3 * 2 * Wg.numel() * Wg.element_size() / t2 / 1e9,
    }


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py measures one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2405_01943_amd as dass
    from paper_2405_01943_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dass.load_library()  # raises if the HIP library is missing
    dev = torch.device("cuda:0")
    cfg = synth.CONFIGS[args.config]
    if args.tokens:
        import dataclasses
        cfg = dataclasses.replace(cfg, tokens=args.tokens, chunk=min(cfg.chunk, args.tokens))
    n_keep, m = (int(v) for v in args.nm.split(":"))
    default_workload = args.config == "llama2_7b" and not args.tokens and (n_keep, m) == (2, 4)
    T, d, I = cfg.tokens, cfg.d, cfg.d_int
    esz = 2 if cfg.dtype == "bf16" else 4

    # ---- synthetic inputs, generated on the device chunk by chunk ----------------------
    X, Wg, Wu, Wd = make_inputs(cfg, dev)
    ws_gate = torch.empty(max(16, dass.nm_workspace_bytes(I, d, "rows")), dtype=torch.uint8, device=dev)
    ws_down = torch.empty(max(16, dass.nm_workspace_bytes(d, I, "cols")), dtype=torch.uint8, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)

    # ---- the timed steps -------------------------------------------------------------------
    ms_per_step, s1_avg, s2_avg, norms = run_steps(cfg, n_keep, m, X, Wg, Wu, Wd, args.steps, args.warmup)
    flops = 4.0 * T * d * I
    s1_tflops = flops / (s1_avg * 1e-3) / 1e12

    # ---- stage 2, launch by launch, on copies rotating through > 256 MB ------------------
    n_copies = max(2, int(320e6 // (Wd.numel() * esz)) + 1)
    bytes_per_matrix = 2.0 * Wd.numel() * esz     # every weight read once and written once
    frac_of_hbm = lambda us: bytes_per_matrix / (us * 1e-6) / 1e9 / PEAK_HBM_GBS

    def cold_nm(W0, norm_axis, group_axis, alpha, nk, mm, ws):
        return cold_launch_us(W0, lambda w: dass.score_mask_nm(w, norms, norm_axis, group_axis, alpha, nk, mm,
                                                               workspace=ws), args.stage2_launches, n_copies)

    cold = {"gate": cold_nm(Wg, "rows", "rows", cfg.alpha_gate_up, n_keep, m, ws_gate),
            "down": cold_nm(Wd, "cols", "cols", cfg.alpha_down, n_keep, m, ws_down)}
    s2_gbs = 3 * bytes_per_matrix / (s2_avg * 1e-3) / 1e9
    cold_call_us = (2 * cold["gate"]["median_us"] + cold["down"]["median_us"]) / 3.0

    # ---- the same matrices at 4:8 (the workload names both patterns): a few whole steps for the in-step
    # figure, then launch by launch ---------------------------------------------------------------
    stage2_48 = None
    if (n_keep, m) != (4, 8) and I % 8 == 0:
        _, _, s2_48, _ = run_steps(cfg, 4, 8, X, Wg, Wu, Wd, max(2, min(args.steps, 5)), 1)
        c48 = {"gate": cold_nm(Wg, "rows", "rows", cfg.alpha_gate_up, 4, 8, ws_gate),
               "down": cold_nm(Wd, "cols", "cols", cfg.alpha_down, 4, 8, ws_down)}
        gbs48 = 3 * bytes_per_matrix / (s2_48 * 1e-3) / 1e9
        stage2_48 = {"kernel": "nm_half_batched_kernel at 4:8: Gate + Up in one launch, Down in a second, "
                               "event to event", "bound": "hbm", "achieved": gbs48, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": gbs48 / PEAK_HBM_GBS, "traffic": None,
                     "in_step_ms_3_matrices": s2_48, "cold_gate_us": c48["gate"], "cold_down_us": c48["down"],
                     "cold_gate_frac": frac_of_hbm(c48["gate"]["median_us"]),
                     "cold_down_frac": frac_of_hbm(c48["down"]["median_us"])}

    # ---- the other reading of the group direction: Gate-Proj with groups of M consecutive INPUT weights
    # (norm along the rows, groups along the columns), launch by launch -----------------------------
    other_reading = {}
    for nk, mm in ((2, 4), (4, 8)):
        c = cold_nm(Wg, "rows", "cols", cfg.alpha_gate_up, nk, mm, ws_gate)
        other_reading[f"gate_{nk}:{mm}"] = dict(c, frac=frac_of_hbm(c["median_us"]))

    # ---- unstructured selection, 50 % of every comparison group, launch by launch -------------
    ws_u = torch.empty(max(16, dass.unstructured_workspace_bytes(I, d, Wg.dtype, "rows", "rows"),
                           dass.unstructured_workspace_bytes(d, I, Wd.dtype, "cols", "cols")),
                       dtype=torch.uint8, device=dev)
    unstructured = {}
    for name, W0, axes, alpha in (("gate", Wg, ("rows", "rows"), cfg.alpha_gate_up),
                                  ("down", Wd, ("cols", "cols"), cfg.alpha_down)):
        c = cold_launch_us(W0, lambda w: dass.score_mask_unstructured(w, norms, axes[0], axes[1], alpha, I // 2,
                                                                      workspace=ws_u),
                           max(6, args.stage2_launches - 4), n_copies)
        unstructured[name] = dict(c, GBps=bytes_per_matrix / (c["median_us"] * 1e-6) / 1e9,
                                  frac=frac_of_hbm(c["median_us"]))
    unstructured["bound"] = "hbm"
    unstructured["bytes_per_matrix"] = bytes_per_matrix
    del ws_u

    # ---- the Wanda metric's input-feature norms over the same tokens (reads X once) ------------
    in_sumsq = torch.empty(d, device=dev)
    in_norms = torch.empty(d, device=dev)
    ws_in = torch.empty(max(16, dass.input_norms_workspace_bytes(T, d)), dtype=torch.uint8, device=dev)
    in_ms = []
    for it in range(5):
        a, b = ev(), ev()
        a.record()
        dass.input_norms(X, in_sumsq, norms_out=in_norms, workspace=ws_in)
        b.record()
        torch.cuda.synchronize()
        if it >= 2:
            in_ms.append(a.elapsed_time(b))
    in_ms = statistics.median(in_ms)
    in_bytes = float(T) * d * esz
    input_norms = {"ms": in_ms, "GBps": in_bytes / (in_ms * 1e-3) / 1e9,
                   "frac_of_hbm_peak": in_bytes / (in_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "bytes": in_bytes}

    # ---- stage 2 for a whole model: all layers x (gate, up, down), batched against one call each ----
    model = None
    if args.model_layers > 0:
        L = args.model_layers
        base = (Wg, Wu, Wd)
        kinds = (("rows", "rows", cfg.alpha_gate_up), ("rows", "rows", cfg.alpha_gate_up), ("cols", "cols", cfg.alpha_down))
        layers = [[w.clone() for w in base] for _ in range(L)]      # > 256 MB from 2 layers on: HBM-honest
        tasks = [(layers[l][k], norms, kinds[k][0], kinds[k][1], kinds[k][2]) for l in range(L) for k in range(3)]
        ws_model = torch.empty(max(16, dass.nm_batched_workspace_bytes(tasks)), dtype=torch.uint8, device=dev)

        def restore():
            for lay in layers:
                for w, w0 in zip(lay, base):
                    w.copy_(w0)

        def timed(fn):
            ts = []
            for _ in range(4):
                restore()
                a, b = ev(), ev()
                a.record()
                fn()
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            return statistics.median(ts[1:])

        def one_by_one():
            for w, n, na, ga, al in tasks:
                dass.score_mask_nm(w, n, na, ga, al, n_keep, m, workspace=ws_model)

        ws_u = torch.empty(max(16, dass.unstructured_workspace_bytes(I, d, Wg.dtype, "rows", "rows"),
                               dass.unstructured_workspace_bytes(d, I, Wd.dtype, "cols", "cols")),
                           dtype=torch.uint8, device=dev)

        def unstructured_half():   # 50 % per comparison group, the paper's default setting
            for w, n, na, ga, al in tasks:
                dass.score_mask_unstructured(w, n, na, ga, al, I // 2, workspace=ws_u)

        # the same calls dealt to four streams of the caller's (a workspace each): the short launches of
        # one matrix's selection run beside the long ones of another's
        side = [torch.cuda.Stream() for _ in range(4)]
        ws_side = [torch.empty_like(ws_u) for _ in side]

        def unstructured_half_4_streams():
            for s in side:
                s.wait_stream(torch.cuda.current_stream())
            for k, (w, n, na, ga, al) in enumerate(tasks):
                dass.score_mask_unstructured(w, n, na, ga, al, I // 2, workspace=ws_side[k % 4], stream=side[k % 4])
            for s in side:
                torch.cuda.current_stream().wait_stream(s)

        ms_batched = timed(lambda: dass.score_mask_nm_batched(tasks, n_keep, m, workspace=ws_model))
        ms_single = timed(one_by_one)
        ms_unstructured = timed(unstructured_half)
        ms_unstructured_4 = timed(unstructured_half_4_streams)
        del ws_side, side
        model_bytes = 3 * L * bytes_per_matrix
        model = {"layers": L, "matrices": 3 * L, "bytes": model_bytes,
                 "batched_ms": ms_batched, "batched_GBps": model_bytes / (ms_batched * 1e-3) / 1e9,
                 "batched_frac_of_hbm_peak": model_bytes / (ms_batched * 1e-3) / 1e9 / PEAK_HBM_GBS,
                 "one_call_per_matrix_ms": ms_single,
                 "one_call_per_matrix_GBps": model_bytes / (ms_single * 1e-3) / 1e9,
                 "unstructured_50pct_ms": ms_unstructured,
                 "unstructured_50pct_GBps": model_bytes / (ms_unstructured * 1e-3) / 1e9,
                 "unstructured_50pct_4_streams_ms": ms_unstructured_4,
                 "unstructured_50pct_4_streams_GBps": model_bytes / (ms_unstructured_4 * 1e-3) / 1e9}
        del layers, tasks

    # ---- pruning blocks one after the other: the pruned MLP's output (Eq. 2 + Eq. 3) over all tokens,
    # and the 2:4 compressed form of the pruned Down-Proj and Gate-Proj ---------------------------
    chain = None
    if args.model_layers > 0 and Wg.dtype == torch.bfloat16 and d % 64 == 0 and I % 64 == 0 and (n_keep, m) == (2, 4):
        pruned = [w.clone() for w in (Wg, Wu, Wd)]
        dass.score_mask_nm(pruned[0], norms, "rows", "rows", cfg.alpha_gate_up, 2, 4, workspace=ws_gate)
        dass.score_mask_nm(pruned[1], norms, "rows", "rows", cfg.alpha_gate_up, 2, 4, workspace=ws_gate)
        dass.score_mask_nm(pruned[2], norms, "cols", "cols", cfg.alpha_down, 2, 4, workspace=ws_down)
        nxt = torch.empty((T, d), dtype=Wg.dtype, device=dev)
        ws_f = torch.empty(dass.mlp_forward_workspace_bytes(T, d, I), dtype=torch.uint8, device=dev)
        f_ms = []
        for it in range(4):
            a, b = ev(), ev()
            a.record()
            dass.mlp_forward(X, pruned[0], pruned[1], pruned[2], cfg.act, nxt, workspace=ws_f)
            b.record()
            torch.cuda.synchronize()
            if it >= 1:
                f_ms.append(a.elapsed_time(b))
        f_ms = statistics.median(f_ms)
        # Eq. 3 alone from the compressed Down-Proj on the sparse MFMA, on the y the forward pass left
        Yb = ws_f.view(Wg.dtype).view(T, I)
        sp_vals = torch.empty((d, I // 2), dtype=Wg.dtype, device=dev)
        sp_meta = torch.empty((d, I // 8), dtype=torch.uint8, device=dev)
        dass.compress_24(pruned[2], "cols", sp_vals, sp_meta)
        sp_ms = []
        for it in range(4):
            a, b = ev(), ev()
            a.record()
            dass.down_proj_sparse24(Yb, sp_vals, sp_meta, nxt)
            b.record()
            torch.cuda.synchronize()
            if it >= 1:
                sp_ms.append(a.elapsed_time(b))
        sp_ms = statistics.median(sp_ms)
        # the pruned block end to end with the compressed Down-Proj: Eq. 2 alone, then the sparse Eq. 3
        fs_ms = []
        for it in range(4):
            a, b = ev(), ev()
            a.record()
            dass.mlp_forward(X, pruned[0], pruned[1], None, cfg.act, None, workspace=ws_f)
            dass.down_proj_sparse24(Yb, sp_vals, sp_meta, nxt)
            b.record()
            torch.cuda.synchronize()
            if it >= 1:
                fs_ms.append(a.elapsed_time(b))
        fs_ms = statistics.median(fs_ms)
        del ws_f, nxt, Yb, sp_vals, sp_meta
        cmp_us = {}
        for name, w, axis in (("down_cols", pruned[2], "cols"), ("gate_rows", pruned[0], "rows")):
            rows, cols = w.shape
            vals = torch.empty((rows // 2, cols) if axis == "rows" else (rows, cols // 2), dtype=w.dtype, device=dev)
            meta = torch.empty((rows // 4, cols // 2) if axis == "rows" else (rows, cols // 8), dtype=torch.uint8,
                               device=dev)
            copies = [w.clone() for _ in range(n_copies)]   # rotate through > 256 MB, as for stage 2
            ts = []
            for it in range(12):
                a, b = ev(), ev()
                a.record()
                dass.compress_24(copies[it % n_copies], axis, vals, meta)
                b.record()
                torch.cuda.synchronize()
                if it >= 4:
                    ts.append(a.elapsed_time(b))
            cmp_us[name] = statistics.median(ts) * 1e3
            del copies, vals, meta
        cmp_bytes = Wd.numel() * (esz + esz / 2.0 + 0.125)   # read W, write half of it and 1 bit per weight
        chain = {"mlp_forward_ms": f_ms, "mlp_forward_TFLOPs": 6.0 * T * d * I / (f_ms * 1e-3) / 1e12,
                 "mlp_forward_frac_of_mfma_peak": 6.0 * T * d * I / (f_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                 "mlp_forward_sparse_down_ms": fs_ms,
                 "mlp_forward_sparse_down_dense_equivalent_TFLOPs": 6.0 * T * d * I / (fs_ms * 1e-3) / 1e12,
                 "down_proj_sparse24_ms": sp_ms,
                 "down_proj_sparse24_dense_equivalent_TFLOPs": 2.0 * T * d * I / (sp_ms * 1e-3) / 1e12,
                 "compress_24_us": cmp_us, "compress_24_bytes": cmp_bytes,
                 "compress_24_GBps": {k: cmp_bytes / (v * 1e-6) / 1e9 for k, v in cmp_us.items()}}
        del pruned

    # ---- every other configuration, a few steps each (their tensors replace this workload's) --------
    others = []
    names = [] if args.other_configs == "none" else \
        [n for n in synth.CONFIGS if n != cfg.name] if args.other_configs == "all" else args.other_configs.split(",")
    x_sample = X[:min(T, 8192)].clone()
    w_cpu = None
    if not args.no_cpu_baseline:
        w_cpu = tuple(w.cpu() for w in (Wg, Wu, Wd))
    norms_cpu = norms.cpu().numpy()
    if names:
        del X
        torch.cuda.empty_cache()
    for name in names:
        oc = synth.CONFIGS[name]
        onk, om = oc.nm[0]
        oX, oWg, oWu, oWd = make_inputs(oc, dev)
        o_ms, o_s1, o_s2, o_norms = run_steps(oc, onk, om, oX, oWg, oWu, oWd, args.other_steps, 1)
        o_esz = 2 if oc.dtype == "bf16" else 4
        o_flops = 4.0 * oc.tokens * oc.d * oc.d_int
        o_bytes = 3 * 2.0 * oWd.numel() * o_esz
        others.append({"name": name, "d": oc.d, "d_int": oc.d_int, "tokens": oc.tokens, "chunk": oc.chunk,
                       "dtype": oc.dtype, "act": oc.act, "nm": f"{onk}:{om}", "steps": args.other_steps,
                       "ms_per_step": o_ms, "tokens_per_s": oc.tokens / (o_ms * 1e-3),
                       "stage1_ms": o_s1, "stage1_TFLOPs": o_flops / (o_s1 * 1e-3) / 1e12,
                       "stage1_frac": (o_flops / (o_s1 * 1e-3) / 1e12 / PEAK_BF16_TFLOPS) if oc.dtype == "bf16" else None,
                       "stage2_us_3_matrices": o_s2 * 1e3, "stage2_GBps": o_bytes / (o_s2 * 1e-3) / 1e9,
                       "stage2_frac": o_bytes / (o_s2 * 1e-3) / 1e9 / PEAK_HBM_GBS})
        if oc.unstructured is not None:   # the configuration's unstructured variant, launch by launch on cold copies
            o_prune = int(round(oc.unstructured * oc.d_int))
            o_mat = 2.0 * oWd.numel() * o_esz
            o_copies = max(2, int(320e6 // (oWd.numel() * o_esz)) + 1)
            o_ws = torch.empty(max(16, dass.unstructured_workspace_bytes(oc.d_int, oc.d, oWg.dtype, "rows", "rows"),
                                   dass.unstructured_workspace_bytes(oc.d, oc.d_int, oWd.dtype, "cols", "cols")),
                               dtype=torch.uint8, device=dev)
            o_u = {"n_prune_per_line": o_prune, "bytes_per_matrix": o_mat}
            for key, W0, axis, alpha in (("gate", oWg, "rows", oc.alpha_gate_up), ("down", oWd, "cols", oc.alpha_down)):
                c = cold_launch_us(W0, lambda w: dass.score_mask_unstructured(w, o_norms, axis, axis, alpha, o_prune,
                                                                              workspace=o_ws), max(6, args.stage2_launches - 4), o_copies)
                o_u[key] = dict(c, GBps=o_mat / (c["median_us"] * 1e-6) / 1e9,
                                frac=o_mat / (c["median_us"] * 1e-6) / 1e9 / PEAK_HBM_GBS)
            others[-1]["unstructured"] = o_u
            del o_ws
        del oX, oWg, oWu, oWd, o_norms
        torch.cuda.empty_cache()

    out = {
        "metric": "calib tokens/s (fused GLU-norm, %MFMA peak) + N:M mask GB/s, LLaMA2-7B MLP",
        "value": T / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}-shaped {cfg.act} MLP, one pass of calibration norms + "
                               f"{n_keep}:{m} DaSS masks of gate/up/down",
                   "d": d, "d_int": I, "tokens": T, "chunk": cfg.chunk, "nm": f"{n_keep}:{m}",
                   "alpha_gate_up": cfg.alpha_gate_up, "alpha_down": cfg.alpha_down},
        "roofline": {"kernel": "calib_pipe64_kernel", "bound": "mfma", "achieved": s1_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": s1_tflops / PEAK_BF16_TFLOPS,
                     "traffic": measured_traffic("stage1", default_workload)},
        "roofline_stage2": {"kernel": "nm_half_batched_kernel: Gate + Up in one launch, Down in a second, "
                                      "event to event", "bound": "hbm", "achieved": s2_gbs,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": s2_gbs / PEAK_HBM_GBS,
                            "traffic": measured_traffic("stage2", default_workload)},
        "stage1": {"ms": s1_avg, "tokens_per_s": T / (s1_avg * 1e-3), "TFLOPs": s1_tflops},
        "stage2": {"in_step_ms_3_matrices": s2_avg, "cold_gate_us": cold["gate"],
                   "cold_down_us": cold["down"], "copies_rotated": n_copies,
                   "cold_single_launch_GBps": bytes_per_matrix / (cold_call_us * 1e-6) / 1e9,
                   "bytes_per_matrix": bytes_per_matrix},
    }
    if stage2_48 is not None:
        out["roofline_stage2_48"] = stage2_48
    out["stage2_other_reading"] = other_reading
    out["unstructured"] = unstructured
    if others:
        out["all_configs"] = others
    out["input_norms_eq1"] = input_norms
    if model is not None:
        out["stage2_whole_model"] = model
    if chain is not None:
        out["layer_chaining"] = chain
    if not args.no_cpu_baseline:   # the first 8192 tokens: about 14 s of the oracle on 16 host threads
        out["cpu_baseline"] = cpu_baseline(cfg, n_keep, m, w_cpu[0], w_cpu[1], w_cpu[2], x_sample, norms_cpu)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
