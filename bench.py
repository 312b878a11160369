#!/usr/bin/env python3
"""Decode-step throughput of the AttentionPredictor hot path on one MI355X.

One step = predict + top-k select + block-sparse decode attention + history push for every
instance of the workload (fused `ap_step`), plus the dense calibration call on every M-th step.
Inputs are synthetic, seeded and resident in HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this file, scaled by what the
# same counters read for ap_stream_copy of known size: one line per (kernel, workload, instances) in this table,
# written from the summaries beside it.  A kernel and shape the table does not hold reports `null`.
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")


def measured_traffic_gb(kernel, workload, n_inst):
    try:
        with open(TRAFFIC_TABLE) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and not line.startswith("#") and parts[0] == kernel and parts[1] == workload \
                        and int(parts[2]) == n_inst:
                    return float(parts[3])
    except (OSError, ValueError):
        pass
    return None


def algorithmic_bytes(w, t):
    """HBM bytes Algorithm 1 itself has to move per instance for one call of each kernel."""
    s_kv = 2 if w.kv_dtype == "bf16" else 4
    nb = (t + w.block - 1) // w.block
    k = min(w.k_blocks, nb)
    return {
        "predict_full": w.hist_len * nb * 4 + nb * 4,
        "predict_incremental": 10 * nb * 4 + 3 * nb * 4,      # 10 history rows, state read + write, pred write
        "select": nb * 4 + k * 4,
        "sparse_decode": 2 * k * w.block * w.head_dim * s_kv + w.g * w.head_dim * (s_kv + 4) + k * 4 + nb * 4,
        "calibrate": t * w.head_dim * s_kv + w.g * w.head_dim * s_kv + nb * 4,
    }


def algorithmic_flops(w, t):
    nb = (t + w.block - 1) // w.block
    k = min(w.k_blocks, nb)
    y1_row, y2_tap_row = 2 * 9 * w.c1, 2 * 3 * w.c1 * w.c2       # flops per column per y1 row / per (y2 row, tap row)
    return {
        "predict_full": (y1_row + 3 * y2_tap_row) * w.hist_len * nb + 2 * w.c2 * nb,
        # 8 y1 rows and 6 y2 rows (two of them with one tap row outside the window) per column
        "predict_incremental": (8 * y1_row + 16 * y2_tap_row) * nb + 6 * 2 * w.c2 * nb,
        "sparse_decode": 4 * w.g * w.head_dim * k * w.block,
    }


def cpu_baseline(w, hist, dev, K, V, budget_s=20.0, max_inst=16):
    """Times the oracle's decode_step as it stands on a bounded sample of instances."""
    import numpy as np
    import torch
    from oracle import attnpred_oracle as orc
    from workloads import predictor_weights, queries, to_f64
    try:
        cores = len(os.sched_getaffinity(0))               # host cores this process may run on
    except AttributeError:
        cores = os.cpu_count() or 1
    wts = orc.PredictorWeights.from_blob(predictor_weights(w), w.c1, w.c2)
    t = w.t_at(0)
    q = queries(w, 0, dev)
    n_done, t_used = 0, 0.0
    for i in range(min(max_inst, w.n_inst, hist.shape[0])):
        h = hist[i].cpu().numpy().astype(np.float64)
        qi, Ki, Vi = to_f64(q[i]), to_f64(K[i]), to_f64(V[i])
        t0 = time.perf_counter()
        orc.decode_step(h, qi, Ki, Vi, t, wts, b=w.block, k=w.k_blocks, n_sink=w.n_sink, n_local=w.n_local,
                        calibrate=False)
        t_used += time.perf_counter() - t0
        n_done += 1
        if t_used > budget_s:
            break
    per_inst = t_used / n_done
    return {
        "value": 1.0 / (per_inst * w.n_inst), "unit": "steps/s", "cores": int(cores), "kind": "oracle",
        "sample": f"{n_done} of {w.n_inst} instances x 1 non-calibration decode step of {w.name}, "
                  f"{per_inst * 1e3:.1f} ms per instance-step, extrapolated to all instances; the oracle is numpy "
                  f"float64 with Python loops over the kernel taps: one thread except inside its matrix products, "
                  f"which may use the BLAS pool on the cores counted",
    }


def main_offload(args):
    """Decode with the K/V cache in pinned host memory: per layer, the next token's selected blocks are gathered
    over PCIe on a second stream while the other layers compute.  Reported beside it: the time a dense-attention
    offload scheme needs just to move the whole cache to the device once per token (its lower bound)."""
    import torch
    from paper_2502_04077_amd.offload import OffloadRun
    from workloads import CONFIGS, kv_cache, predictor_weights, queries

    steps = min(args.steps, 128)
    total_steps = args.warmup + steps
    w = CONFIGS["cfg1"].with_(name="cfg1x32-offload" + ("-planted" if args.planted else ""), layers=32,
                              steps=total_steps, planted=args.planted)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K, V = kv_cache(w, dev)
    K_host = torch.empty(K.shape, dtype=K.dtype, pin_memory=True)
    V_host = torch.empty(V.shape, dtype=V.dtype, pin_memory=True)
    K_host.copy_(K)
    V_host.copy_(V)
    first = w.t_at(0) - 1                                  # index of the first decoded token
    k_new = K[:, first:first + total_steps, :].transpose(0, 1).contiguous()   # [step][n_inst][d]
    v_new = V[:, first:first + total_steps, :].transpose(0, 1).contiguous()
    del K, V
    torch.cuda.empty_cache()
    run = OffloadRun(w, K_host, V_host, dev)
    run.set_weights(predictor_weights(w))
    H = w.hist_len
    for j in range(H):
        run.warmup_calibrate(queries(w, j - H, dev), w.t0 - H + 1 + j)
    qs = [queries(w, s, dev) for s in range(total_steps)]
    run.start(w.t_at(0))
    torch.cuda.synchronize()

    def one_step(s, calib=None):
        run.step(qs[s], k_new[s], v_new[s], w.t_at(s), calibrate=w.is_calibration_step(s) if calib is None else calib)

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    fetched0 = run.blocks_fetched()
    t0 = time.perf_counter()
    for s in range(args.warmup, total_steps):
        one_step(s)
    issued = time.perf_counter() - t0                      # host time to enqueue the steps
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    n_calib = sum(1 for s in range(args.warmup, total_steps) if w.is_calibration_step(s))
    run.finish()
    ms_per_step = elapsed * 1e3 / steps
    fetched = run.blocks_fetched() - fetched0              # blocks that actually crossed the link

    # The dense alternative must at least bring every K and V row to the device once per token.
    esize = K_host.element_size()
    t_mid = w.t_at(args.warmup + steps // 2)
    layer_rows = run.ipl
    stage = torch.empty((layer_rows, w.t_cap, w.head_dim), dtype=K_host.dtype, device=dev)
    for rep in range(2):
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for l in range(w.layers):
            stage.copy_(K_host[l * layer_rows:(l + 1) * layer_rows], non_blocking=True)
            stage.copy_(V_host[l * layer_rows:(l + 1) * layer_rows], non_blocking=True)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - c0) * 1e3
    dense_bytes = 2 * w.n_inst * w.t_cap * w.head_dim * esize
    block_bytes = 2 * w.block * w.head_dim * esize         # K and V
    selected_bytes = w.n_inst * w.k_blocks * block_bytes   # per step, were every selected block fetched
    staged_bytes = fetched * block_bytes / steps           # per step, fetched in fact (blocks that stay selected are kept)
    calib_bytes = w.n_inst * t_mid * w.head_dim * esize
    out = {
        "metric": "decode steps/s with the K/V cache in host memory (cross-token prefetch of the selected blocks)",
        "value": 1e3 / ms_per_step, "unit": "steps/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "host_enqueue_ms_per_step": issued * 1e3 / steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "instances": w.n_inst, "layers": w.layers, "batch": w.batch,
                   "kv_heads": w.kv_heads, "q_per_kv": w.g, "head_dim": w.head_dim, "context": w.t0, "block": w.block,
                   "history": w.hist_len, "budget_tokens": w.budget_tokens, "predictor_channels": [w.c1, w.c2],
                   "calibration_every": w.calib_every, "calibration_steps_in_timed_region": n_calib,
                   "kv_cache": "pinned host memory", "host_cache_GB": dense_bytes / 1e9},
        "pcie": {"selected_MB_per_step": selected_bytes / 1e6, "fetched_MB_per_step": staged_bytes / 1e6,
                 "fetched_fraction_of_selected": staged_bytes / selected_bytes,
                 "calibration_MB_per_step_amortised": calib_bytes * n_calib / steps / 1e6,
                 "achieved_GBs": (staged_bytes * steps + calib_bytes * n_calib) / elapsed / 1e9},
        "dense_offload_transfer": {"ms_per_token": dense_ms, "GBs": dense_bytes / dense_ms / 1e6,
                                   "what": "hipMemcpyAsync of the whole K and V cache to the device, no compute"},
        "speedup_vs_dense_transfer": dense_ms / ms_per_step,
    }
    print(json.dumps(out))


def main():
    ap_ = argparse.ArgumentParser()
    ap_.add_argument("--gpus", type=int, default=1)
    ap_.add_argument("--steps", type=int, default=512)
    ap_.add_argument("--warmup", type=int, default=8)
    ap_.add_argument("--workload", default="cfg2", help="cfg0..cfg4 (default: cfg2, the 32-layer batch-8 32K case)")
    ap_.add_argument("--no-cpu-baseline", action="store_true")
    ap_.add_argument("--no-breakdown", action="store_true")
    ap_.add_argument("--offload", action="store_true",
                     help="K/V in pinned host memory with cross-token prefetching (Sec. 3.4); one 8B-shaped model, "
                          "batch 1, 32 layers, 32K context; prints its own JSON line")
    ap_.add_argument("--no-dense-figure", action="store_true",
                     help="skip the launches of the attention kernel over the whole context (they share the sparse "
                          "kernel's name in a profile)")
    ap_.add_argument("--refresh-every", type=int, default=1,
                     help="re-make the selection on every N-th step only and carry it over in between (Sec. 3.3)")
    ap_.add_argument("--dense-layers", type=int, default=0,
                     help="the first N layers attend to the whole cache in every step (Sec. 4.1 keeps two uncompressed)")
    ap_.add_argument("--predictor-channels", type=int, nargs=2, metavar=("C1", "C2"), default=None,
                     help="hidden channels of the predictor instead of the workload's (16 32 is the paper's own network)")
    ap_.add_argument("--planted", action="store_true",
                     help="with --offload: keys and queries with the planted sink / stripe / local / slash structure of "
                          "cfg4 instead of plain Gaussian ones")
    args = ap_.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only; --gpus must be 1 (instances are independent, "
              "sharding across GPUs is not built).", file=sys.stderr)
        sys.exit(2)

    if args.offload:
        return main_offload(args)

    import torch
    from paper_2502_04077_amd.runner import DecodeRun, DenseRun
    from workloads import CONFIGS, kv_cache, predictor_weights, queries

    w_all = CONFIGS[args.workload]
    total_steps = args.warmup + args.steps
    if total_steps > w_all.steps:
        w_all = w_all.with_(steps=total_steps)
    if args.predictor_channels:
        w_all = w_all.with_(c1=args.predictor_channels[0], c2=args.predictor_channels[1])
    if not 0 <= args.dense_layers < w_all.layers:
        print("bench.py: --dense-layers must leave at least one sparse layer", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    K_all, V_all = kv_cache(w_all, dev)
    # Instances are layer-major: the dense layers are the first nd instances, everything below is the sparse rest.
    nd = args.dense_layers * w_all.batch * w_all.kv_heads
    w = w_all.with_(layers=w_all.layers - args.dense_layers)
    K, V = K_all[nd:], V_all[nd:]
    dense = DenseRun(w_all, args.dense_layers, dev) if nd else None
    run = DecodeRun(w, dev, refresh_every=args.refresh_every)
    run.set_weights(predictor_weights(w))
    H = w.hist_len
    # Every input is drawn before the history warm-up, so that nothing but the decode calls themselves lies between
    # that warm-up (H dense passes over the K cache) and the timed steps.
    qs_all = [queries(w_all, s, dev) for s in range(total_steps)]
    qs = [q[nd:] for q in qs_all]
    qs_warm = [queries(w_all, j - H, dev)[nd:] for j in range(H)]
    torch.cuda.synchronize()
    for j in range(H):                                    # prefill tail fills the history
        run.warmup_calibrate(qs_warm[j], K, w.t0 - H + 1 + j)
    # The CPU baseline (below) starts from this history: the ring slots of the first instances are copied on the
    # stream (no host synchronisation, no large temporary: an idle GPU takes tens of milliseconds to clock up
    # again) and put into window order on the host later.
    ring0, n_pushed0 = run.hist[: min(16, w.n_inst)].clone(), run.n_pushed

    modes = []

    def one_step(s):
        if dense is not None:
            dense.step(qs_all[s][:nd], K_all[:nd], V_all[:nd], w.t_at(s))
        return run.step(qs[s], K, V, w.t_at(s), calibrate=w.is_calibration_step(s))

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    del qs_warm
    t0 = time.perf_counter()
    for s in range(args.warmup, total_steps):
        modes.append(one_step(s) == 0)       # mode 0 = full-tile re-base
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    n_calib = sum(1 for s in range(args.warmup, total_steps) if w.is_calibration_step(s))
    n_rebase = sum(modes)

    # Per-call durations with events on the launch stream, replaying the same steps un-fused.
    kern_ms = {}
    if not args.no_breakdown:
        from paper_2502_04077_amd import AP_PRED_ADVANCE, AP_PRED_REBASE
        ev = lambda: torch.cuda.Event(enable_timing=True)
        marks = {}

        def timed(name, fn):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            marks.setdefault(name, []).append((a, b))

        for s in range(args.warmup, total_steps):
            t = w.t_at(s)
            nb = run.nb(t)
            mode = run._pred_mode(t)
            pname = {AP_PRED_ADVANCE: "predict_incremental", AP_PRED_REBASE: "predict_full"}.get(mode, "predict_hold")
            if nb != run.nb(t - 1) and mode == AP_PRED_ADVANCE:
                pname = "predict_incremental_grow"
            timed(pname, lambda: run.ctx.predict_incremental(run.hist, run.n_pushed, nb, run.nb(t - 1), mode,
                                                             run.pstate, run.pred, run.ws))
            run.state_n, run.state_t = run.n_pushed, t
            timed("select", lambda: run.ctx.select_topk(run.pred, nb, run.idx, run.cnt, run.ws))
            timed("sparse_decode", lambda: run.ctx.sparse_decode(qs[s], K, V, t, run.idx, run.cnt, run.out, run.row, run.ws))
            if w.is_calibration_step(s):
                timed("calibrate", lambda: run.ctx.calibrate(qs[s], K, t, run.row, run.ws))
            timed("update_history", lambda: run.ctx.update_history(run.hist, run.n_pushed, run.row))
            run.n_pushed += 1
        calib_outside = "calibrate" not in marks
        if calib_outside:                                  # no calibration step fell into the replayed steps: time one
            t_c = w.t_at(total_steps - 1)
            run.ctx.calibrate(qs[-1], K, t_c, run.row, run.ws)
            for _ in range(2):
                timed("calibrate", lambda: run.ctx.calibrate(qs[-1], K, t_c, run.row, run.ws))
        torch.cuda.synchronize()
        for n, m in marks.items():
            kern_ms[n] = sum(a.elapsed_time(b) for a, b in m) / len(m)
        kern_ms = {k: round(v, 5) for k, v in kern_ms.items()}

    # Attention over the whole cache with the same kernel (a budget of all blocks), for the sparse-versus-dense ratio.
    dense_ms = None
    if not args.no_breakdown and not args.no_dense_figure:
        full = DenseRun(w_all, w_all.layers, dev)
        t_d = w.t_at(args.warmup + args.steps // 2)
        full.step(qs_all[0], K_all, V_all, t_d)
        torch.cuda.synchronize()
        d0, d1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        d0.record()
        for _ in range(3):
            full.step(qs_all[0], K_all, V_all, t_d)
        d1.record()
        torch.cuda.synchronize()
        dense_ms = d0.elapsed_time(d1) / 3
        del full
        torch.cuda.empty_cache()

    # Read bandwidth this machine reaches with a plain streaming kernel over the K cache (same run).
    from paper_2502_04077_amd import stream_read
    sink = torch.zeros((65536 * 16,), dtype=torch.uint8, device=dev)
    span = K.view(-1)[: min(K.numel(), 4 * 2**30)]                 # up to 8 GiB of bf16
    stream_read(span, sink, 4096)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        stream_read(span, sink, 4096)
    e1.record()
    torch.cuda.synchronize()
    ceiling_gbs = span.numel() * span.element_size() * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    # One plain copy of known size (1 GiB read + 1 GiB written): the reference dispatch for counter scaling.
    from paper_2502_04077_amd import stream_copy
    copy_src = K.view(-1)[: 2**29]
    copy_dst = torch.empty_like(copy_src)
    stream_copy(copy_src, copy_dst, 4096)
    torch.cuda.synchronize()
    del copy_dst

    # The oracle on the host cores, after everything that is timed on the GPU: the GPU idles meanwhile, and
    # whatever runs right after an idle spell runs at low clocks.
    cpu = None
    if not args.no_cpu_baseline:
        slots = [(n_pushed0 - H + r) % run.R for r in range(H)]          # (n_pushed0 >= H after the warm-up)
        cpu = cpu_baseline(w, ring0[:, slots, :], run.dev, K, V)

    t_mid = w.t_at(args.warmup + args.steps // 2)
    ab = algorithmic_bytes(w, t_mid)
    af = algorithmic_flops(w, t_mid)
    roofline = None
    if kern_ms:
        per_step = {k: v for k, v in kern_ms.items() if k in ("predict_incremental", "select", "sparse_decode")}
        dom = max(per_step, key=per_step.get)
        ach = ab[dom] * w.n_inst / (kern_ms[dom] * 1e-3) / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBS,
                    # (the table's predictor line was measured with the 8/8 network)
                    "traffic": (measured_traffic_gb(dom, w.name, w.n_inst)
                                if dom != "predict_incremental" or (w.c1, w.c2) == (8, 8) else None),
                    "avg_launch_ms": kern_ms[dom], "algorithmic_GB_per_launch": ab[dom] * w.n_inst / 1e9,
                    "measured_read_ceiling_GBs": ceiling_gbs, "frac_of_measured_ceiling": ach / ceiling_gbs}
        if dom == "predict_incremental":
            # With the larger networks the predictor is the longest per-step kernel, and it is bound by arithmetic:
            # the dense f16 MFMA peak where both layers run on MFMA, else the fp32 vector rate without packed
            # instructions (256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz).
            mfma_pred = run.ctx.cfg.flags == 0 and (w.c1, w.c2) in ((8, 8), (16, 32))
            peak = 2500.0 if mfma_pred else 78.6
            tf = af[dom] * w.n_inst / (kern_ms[dom] * 1e-3) / 1e12
            roofline.update({"bound": "mfma" if mfma_pred else "alu", "achieved": tf, "peak": peak, "unit": "TFLOP/s",
                             "frac": tf / peak, "algorithmic_GFLOP_per_launch": af[dom] * w.n_inst / 1e9,
                             "hbm_GBs": ach})
            roofline.pop("frac_of_measured_ceiling")
        roofline["other_kernels"] = {
            k: {"bound": "hbm", "GB/s": ab[k] * w.n_inst / (kern_ms[k] * 1e-3) / 1e9,
                "frac": ab[k] * w.n_inst / (kern_ms[k] * 1e-3) / 1e9 / HBM_PEAK_GBS, "avg_launch_ms": kern_ms[k]}
            for k in ("calibrate", "predict_incremental", "select") if k in kern_ms and k != dom}
    step_bytes = (ab["predict_incremental"] + ab["select"] + ab["sparse_decode"]) * w.n_inst
    timed_bytes = step_bytes * args.steps + ab["calibrate"] * w.n_inst * n_calib + ab["predict_full"] * w.n_inst * n_rebase
    mfma = run.ctx.cfg.flags == 0 and (w.c1, w.c2) in ((8, 8), (16, 32))
    out = {
        "metric": "predict+top-k+sparse-attn decode steps/s at 32K ctx; % HBM peak",
        "value": 1e3 / ms_per_step, "unit": "steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.kv_dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "instances": w_all.n_inst, "layers": w_all.layers, "batch": w.batch,
                   "kv_heads": w.kv_heads, "q_per_kv": w.g, "head_dim": w.head_dim, "context": w.t0,
                   "block": w.block, "history": w.hist_len, "budget_tokens": w.budget_tokens,
                   "predictor_channels": [w.c1, w.c2], "calibration_every": w.calib_every,
                   "calibration_steps_in_timed_region": n_calib, "predictor": "incremental",
                   "predictor_arith": ("f16 MFMA operands (history and first-layer maps as differences from the "
                                       "all-zero-history response), fp32 accumulate" if mfma else "fp32 FMA"),
                   "predictor_rebase_every": run.rebase_every, "rebase_steps_in_timed_region": n_rebase,
                   "selection_refresh_every": args.refresh_every, "dense_layers": args.dense_layers},
        # the per-step calls only (predict + select + sparse decode): their algorithmic bytes over the wall time of
        # the whole timed region, whatever else ran in it ...
        "step_hbm_frac": step_bytes * args.steps / elapsed / 1e9 / HBM_PEAK_GBS,
        "step_algorithmic_GB": step_bytes / 1e9,
        # ... and with the bytes of the calibrations and re-bases that fell into the region counted as well
        "step_hbm_frac_with_calibration": timed_bytes / elapsed / 1e9 / HBM_PEAK_GBS,
        "kernel_ms": kern_ms,
        "calibrate_timed_outside_region": bool(kern_ms) and calib_outside,
        # the same attention kernel over every block of the context (all instances), and what the budget saves
        "dense_attention": None if dense_ms is None else {
            "ms": dense_ms, "GBs": 2 * w_all.n_inst * t_mid * w_all.head_dim * (2 if w_all.kv_dtype == "bf16" else 4) / dense_ms / 1e6,
            "sparse_decode_speedup": dense_ms / (kern_ms["sparse_decode"] * w_all.n_inst / w.n_inst) if kern_ms else None},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
