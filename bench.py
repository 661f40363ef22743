#!/usr/bin/env python3
"""Benchmark of the LASNet sparse-bottleneck hot path on one MI355X.

One "step" = the whole path over one synthetic batch that is already resident in HBM:
lasnet_masker_ex (pool -> logit -> threshold -> index list, inactive cells passed through to
out) followed by lasnet_sparse_bottleneck_ex (gather + conv1 / conv3x3 / conv3 + scatter-add
on the active cells), with the active-patch count staying on the device.  Every element of
out is written in every step.  Default workload: ResNet-101 stage-3
bottleneck, 14x14x1024, mid 256, S=2, batch 128, bf16, masker calibrated to r = 0.5.

Prints ONE JSON line: whole-job images/s, plus
  roofline      the fused bottleneck kernel against the bf16 MFMA peak on ACTIVE FLOPs
                (r * N * H*W * 34*M^2; halo recompute is never credited), its duration
                measured here with events on the launch stream;
  cpu_baseline  the numpy fp64 oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# Bytes per launch of the fused kernel between L2 and the memory side, from two rocprofv3 --pmc
# runs (FETCH_SIZE, WRITE_SIZE), each scaled by what the same counter reads for the library's
# plain copy kernel of known size (profiles/bench_<workload>_hbm_traffic_pmc.txt).
MEASURED_TRAFFIC_BYTES = {"stage3_b128": 113952097, "stage1_b64": 96091086}   # at the workload's own ratio


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="stage3_b128",
                    help="stage3_b128 (headline) | stage2_b128 | stage1_b64 | stage4_b128 | stage3_b1")
    ap.add_argument("--ratio", type=float, default=None, help="activation ratio (default: the workload's)")
    ap.add_argument("--nbuf", type=int, default=6,
                    help="distinct x/out buffer pairs rotated over, so that steps see HBM-cold data")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-torch-dense", action="store_true")
    ap.add_argument("--granularity", action="store_true",
                    help="also time the path at every patch size S that divides H and has a matrix-core kernel "
                         "(the latency-ratio-against-S curve of Sec. 4.2 on this GPU)")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the block alone over r in {0.1,.25,.5,.75,1} (index lists fed directly)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by image with no exchange: "
              "each GPU would run its own images). --gpus %d is not supported." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2210_06223_amd import binding as B
    from paper_2210_06223_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(2)
    B.lib()  # fail loudly if the library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    cfg = synth.CONFIGS[args.workload]
    if args.ratio is not None:
        cfg = cfg.with_(r=args.ratio)
    inp = synth.make_block_inputs(cfg, want_f64=False)

    def to_dev(k, v):
        if cfg.dtype == "bf16" and k in ("x", "W1", "W2", "W3"):
            return torch.from_numpy(v.view(np.int16)).view(torch.bfloat16).to(dev)
        return torch.from_numpy(v).to(dev)

    d = {k: to_dev(k, v) for k, v in inp.dev.items()}
    w = (d["W1"], d["b1"], d["W2"], d["b2"], d["W3"], d["b3"])
    S, P = cfg.S, cfg.P

    # Masker bias for the target ratio, calibrated from the library's own fp64 logits.
    logits0 = B.lasnet_masker_logits(d["x"], d["Wm"], 0.0, S).cpu().numpy()
    k_target = int(round(cfg.r * P))
    bm, margin = synth.bias_for_count(logits0, k_target)

    nbuf = max(1, args.nbuf)
    xs = [d["x"]] + [d["x"].clone() for _ in range(nbuf - 1)]
    outs = [torch.empty_like(d["x"]) for _ in range(nbuf)]
    mask = torch.empty((cfg.N, cfg.G, cfg.GW), dtype=torch.uint8, device=dev)
    idx = torch.empty((P,), dtype=torch.int32, device=dev)
    count = torch.zeros((1,), dtype=torch.int32, device=dev)

    def step(i):
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker_ex(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count, pass_out=out)
        B.lasnet_sparse_bottleneck(x, idx, count, S, *w, out=out, flags=B.LASNET_SKIP_IDENTITY)

    def step_separate_copy(i):       # the two spec calls as they are: identity copy inside the block call
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count)
        B.lasnet_sparse_bottleneck(x, idx, count, S, *w, out=out)

    packed = None
    if cfg.dtype == "bf16" and B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, S) == 1:
        packed = B.lasnet_pack_weights(S, d["W1"], d["W2"], d["W3"])   # once, like BN folding

    def step_packed(i):
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker_ex(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count, pass_out=out)
        B.lasnet_sparse_bottleneck_packed(x, idx, count, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=out,
                                          flags=B.LASNET_SKIP_IDENTITY)

    def run_steps(fn):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fn(i)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    dt_packed = run_steps(step_packed) if packed is not None else None
    dt_separate = run_steps(step_separate_copy)
    dt = run_steps(step)
    ms_per_step = dt / args.steps * 1e3
    images_per_s = cfg.N * args.steps / dt
    n_active = int(count.item())

    # ---- per-kernel durations, events on the launch stream (torch's current stream) ----
    def timed(fn, reps):
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for i in range(reps):
            ev[i][0].record()
            fn(i)
            ev[i][1].record()
        torch.cuda.synchronize()
        t = sorted(a.elapsed_time(b) for a, b in ev)
        return {"mean_ms": float(np.mean(t)), "median_ms": t[len(t) // 2], "p10_ms": t[len(t) // 10],
                "p90_ms": t[(len(t) * 9) // 10]}

    def timed_loop(fn, n):
        """Mean duration of n back-to-back calls (one event pair around all of them), in ms."""
        for i in range(5):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n

    reps = max(20, min(args.steps, 200))
    # the fused kernel alone: same launch as inside the step, identity copy skipped (outs already hold x)
    if packed is not None:
        fused_t = timed(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[i % nbuf], idx, count, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf],
            flags=B.LASNET_SKIP_IDENTITY), reps)
    else:
        fused_t = timed(lambda i: B.lasnet_sparse_bottleneck(xs[i % nbuf], idx, count, S, *w, out=outs[i % nbuf],
                                                             flags=B.LASNET_SKIP_IDENTITY), reps)
    if packed is not None:
        fused_loop_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[i % nbuf], idx, count, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf],
            flags=B.LASNET_SKIP_IDENTITY), reps)
    else:
        fused_loop_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck(
            xs[i % nbuf], idx, count, S, *w, out=outs[i % nbuf], flags=B.LASNET_SKIP_IDENTITY), reps)
    # warm regime: the same buffers every launch (x and out may stay in the 256 MB Infinity Cache)
    if packed is not None:
        fused_warm_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[0], idx, count, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[0],
            flags=B.LASNET_SKIP_IDENTITY), reps)
    else:
        fused_warm_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck(
            xs[0], idx, count, S, *w, out=outs[0], flags=B.LASNET_SKIP_IDENTITY), reps)
    block_t = timed(lambda i: B.lasnet_sparse_bottleneck(xs[i % nbuf], idx, count, S, *w, out=outs[i % nbuf]), reps)
    masker_t = timed(lambda i: B.lasnet_masker(xs[i % nbuf], d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count), reps)
    masker_ex_t = timed(lambda i: B.lasnet_masker_ex(xs[i % nbuf], d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count,
                                                     pass_out=outs[i % nbuf]), reps)
    dense_t = timed(lambda i: B.lasnet_dense_bottleneck(xs[i % nbuf], *w, out=outs[i % nbuf]), reps)
    # the dense block through the prepacked entry: every cell active (idx = NULL) on the tile side that
    # lasnet_dense_bottleneck picks (the largest built S that divides H and W)
    dense_packed_ms = None
    if packed is not None:
        S_dense = max(s_ for s_ in range(1, 17) if cfg.H % s_ == 0 and cfg.W % s_ == 0
                      and B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, s_) == 1)
        packed_dense = B.lasnet_pack_weights(S_dense, d["W1"], d["W2"], d["W3"])
        dense_packed_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[i % nbuf], None, None, S_dense, cfg.M, packed_dense, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf]), reps)

    torch_dense = None
    if not args.no_torch_dense and cfg.dtype == "bf16":
        try:
            import torch.nn.functional as F
            W1c = d["W1"][:, :, None, None].contiguous(memory_format=torch.channels_last)
            W2c = d["W2"].permute(0, 3, 1, 2)            # [M,M,3,3] view, channels-last strides
            W3c = d["W3"][:, :, None, None].contiguous(memory_format=torch.channels_last)
            b1c, b2c, b3c = (d[k].to(torch.bfloat16) for k in ("b1", "b2", "b3"))

            def torch_block(i):
                xin = xs[i % nbuf].permute(0, 3, 1, 2)   # NCHW view of NHWC memory
                y = F.relu(F.conv2d(xin, W1c, b1c))
                y = F.relu(F.conv2d(y, W2c, b2c, padding=1))
                return xin + F.conv2d(y, W3c, b3c)

            with torch.no_grad():
                for i in range(5):
                    torch_block(i)
                torch.cuda.synchronize()
                torch_dense = timed(torch_block, reps)
        except Exception as e:  # the yardstick is optional
            torch_dense = {"error": repr(e)[:200]}

    flops_img = cfg.H * cfg.W * (2 * cfg.C * cfg.M + 18 * cfg.M * cfg.M + 2 * cfg.M * cfg.C)
    active_flops = n_active * S * S * (flops_img / (cfg.H * cfg.W))
    fused_s = fused_loop_ms * 1e-3             # average launch duration over `reps` back-to-back launches
    achieved_tflops = active_flops / fused_s / 1e12
    esize = 2 if cfg.dtype == "bf16" else 4
    x_bytes = cfg.N * cfg.H * cfg.W * cfg.C * esize
    # Algorithmic bytes of one launch of the block kernel: every pixel some active patch's (S+2)x(S+2)
    # window holds, read once; the active pixels written once; the weights once.
    m_act = mask.cpu().numpy().astype(bool).reshape(cfg.N, cfg.G, cfg.GW)
    pix_act = np.repeat(np.repeat(m_act, S, axis=1), S, axis=2)
    pad = np.pad(pix_act, ((0, 0), (1, 1), (1, 1)))
    pix_need = np.zeros_like(pix_act)
    for dy in range(3):
        for dx in range(3):
            pix_need |= pad[:, dy:dy + cfg.H, dx:dx + cfg.W]
    w_bytes = (2 * cfg.C * cfg.M + 9 * cfg.M * cfg.M) * esize
    alg_bytes = (int(pix_need.sum()) + int(pix_act.sum())) * cfg.C * esize + w_bytes
    achieved_gbs = alg_bytes / fused_s / 1e9
    kernel_name = ("bottleneck_generic_kernel" if packed is None else
                   "stream_bneck_kernel" if (cfg.C, cfg.M, S) == (256, 64, 8) else "fused_bneck_kernel")
    # the bound is whichever ideal time is longer: active FLOPs at the MFMA peak or these bytes at the HBM peak
    hbm_bound = alg_bytes / (PEAK_HBM_GBS * 1e9) > active_flops / (PEAK_BF16_TFLOPS * 1e12)
    dense_best = dense_t["mean_ms"] if dense_packed_ms is None else dense_packed_ms
    if torch_dense and "mean_ms" in torch_dense:
        dense_best = min(dense_best, torch_dense["mean_ms"])

    sweep = None
    if args.sweep:
        # latency against the activation ratio (index lists fed directly; per-image ratios Beta-distributed
        # around the mean): block = pack + fused kernel on the active cells (the inactive ones are the
        # masker's pass-through, not in this call), against the dense block through the same entry style
        sweep = []
        dense_loop = timed_loop(lambda i: B.lasnet_dense_bottleneck(xs[i % nbuf], *w, out=outs[i % nbuf]), 50)
        if torch_dense and "mean_ms" in torch_dense:
            dense_loop = min(dense_loop, torch_dense["mean_ms"])
        for r in (0.1, 0.25, 0.5, 0.75, 1.0):
            for structure in ("iid", "blob"):
                il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, r, seed=cfg.seed, structure=structure)
                idx_r = torch.zeros((P,), dtype=torch.int32, device=dev)
                idx_r[: len(il)] = torch.from_numpy(il).to(dev)
                cnt_r = torch.tensor([len(il)], dtype=torch.int32, device=dev)
                t_skip = timed_loop(lambda i: B.lasnet_sparse_bottleneck(
                    xs[i % nbuf], idx_r, cnt_r, S, *w, out=outs[i % nbuf], flags=B.LASNET_SKIP_IDENTITY), 50)
                t_copy = timed_loop(lambda i: B.lasnet_sparse_bottleneck(
                    xs[i % nbuf], idx_r, cnt_r, S, *w, out=outs[i % nbuf]), 50)
                sweep.append({"r_mean": r, "structure": structure, "active": len(il),
                              "block_ms": t_skip, "block_with_identity_copy_ms": t_copy,
                              "latency_ratio_vs_dense": t_skip / dense_loop})
        sweep_note = {"dense_ms": dense_loop, "timing": "mean over 50 back-to-back launches between two events"}

    gran = None
    if args.granularity and packed is not None:
        gran = []
        dense_ms = dense_packed_ms
        for S_g in range(1, cfg.H + 1):
            if cfg.H % S_g or cfg.W % S_g or B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, S_g) != 1:
                continue
            Pg = cfg.N * (cfg.H // S_g) * (cfg.W // S_g)
            lg0 = B.lasnet_masker_logits(d["x"], d["Wm"], 0.0, S_g).cpu().numpy()
            bm_g, _ = synth.bias_for_count(lg0, int(round(cfg.r * Pg)))
            mask_g = torch.empty((cfg.N, cfg.H // S_g, cfg.W // S_g), dtype=torch.uint8, device=dev)
            idx_g = torch.empty((Pg,), dtype=torch.int32, device=dev)
            cnt_g = torch.zeros((1,), dtype=torch.int32, device=dev)
            packed_g = B.lasnet_pack_weights(S_g, d["W1"], d["W2"], d["W3"])

            def step_g(i):
                B.lasnet_masker_ex(xs[i % nbuf], d["Wm"], bm_g, S_g, 0.0, mask=mask_g, idx=idx_g, count=cnt_g,
                                   pass_out=outs[i % nbuf])
                B.lasnet_sparse_bottleneck_packed(xs[i % nbuf], idx_g, cnt_g, S_g, cfg.M, packed_g, d["b1"], d["b2"],
                                                  d["b3"], out=outs[i % nbuf], flags=B.LASNET_SKIP_IDENTITY)

            t_step = timed_loop(step_g, 50)
            t_block = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
                xs[i % nbuf], idx_g, cnt_g, S_g, cfg.M, packed_g, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf],
                flags=B.LASNET_SKIP_IDENTITY), 50)
            gran.append({"S": S_g, "cells": Pg, "active": int(cnt_g.item()), "step_ms": t_step, "block_ms": t_block,
                         "latency_ratio_vs_dense_block": t_block / dense_ms,
                         "latency_ratio_step_vs_dense_block": t_step / dense_ms})

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, inp, bm)

    result = {
        "metric": "sparse bottleneck images/s at r=%.2g (masker + index list + identity pass-through + fused block)" % cfg.r,
        "value": images_per_s,
        "unit": "images/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": "%s: ResNet-101 bottleneck %dx%dx%d mid %d, S=%d, batch %d, r=%.3f (%d of %d patches)"
                   % (cfg.name, cfg.H, cfg.W, cfg.C, cfg.M, S, cfg.N, n_active / P, n_active, P),
                   "buffers_rotated": nbuf, "masker_margin": margin},
        "active_tflops_whole_step": active_flops / (ms_per_step * 1e-3) / 1e12,
        "prepacked_weights": None if dt_packed is None else {
            "ms_per_step": dt_packed / args.steps * 1e3, "images_per_s": cfg.N * args.steps / dt_packed,
            "note": "same step through lasnet_sparse_bottleneck_packed (weights repacked once, outside the loop)"},
        "separate_identity_copy": {
            "ms_per_step": dt_separate / args.steps * 1e3, "images_per_s": cfg.N * args.steps / dt_separate,
            "note": "lasnet_masker + lasnet_sparse_bottleneck: the block call copies x to out before the fused kernel"},
        "speedup_vs_dense": dense_best / (fused_loop_ms if packed is not None else block_t["mean_ms"]),
        "speedup_vs_dense_note": "dense block (the faster of the library's and torch/MIOpen's) / sparse block at this r, "
                                 "both without the identity pass-through, which lives in the masker call",
        "kernels_ms": {"masker+compaction": masker_t, "masker+identity+compaction": masker_ex_t,
                       "pack+copy+fused_block": block_t, "fused_block": fused_t,
                       "dense_own": dense_t, "dense_own_prepacked_loop_ms": dense_packed_ms,
                       "fused_block_loop_ms": fused_loop_ms, "fused_block_warm_loop_ms": fused_warm_ms, "dense_torch_miopen": torch_dense},
        "hbm_floor_ms": 2 * x_bytes / (PEAK_HBM_GBS * 1e9) * 1e3,
        "roofline": {"bound": "hbm" if hbm_bound else "mfma", "kernel": kernel_name,
                     "achieved": achieved_gbs if hbm_bound else achieved_tflops,
                     "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
                     "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": achieved_gbs / PEAK_HBM_GBS if hbm_bound else achieved_tflops / PEAK_BF16_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(cfg.name) if args.ratio is None else None,
                     "active_flops_per_launch": active_flops, "algorithmic_bytes_per_launch": alg_bytes,
                     "frac_of_mfma_peak": achieved_tflops / PEAK_BF16_TFLOPS,
                     "frac_of_hbm_peak": achieved_gbs / PEAK_HBM_GBS,
                     "avg_launch_ms": fused_loop_ms,
                     "avg_launch_ms_single_event_pairs": fused_t["mean_ms"], "launches_timed": reps},
        "cpu_baseline": cpu,
    }
    if gran is not None:
        result["granularity_sweep"] = gran
        result["granularity_sweep_note"] = ("r = %.2f at every S (masker bias recalibrated per S); prepacked weights; "
                                            "dense block %.4f ms; mean over 50 back-to-back launches" % (cfg.r, dense_packed_ms))
    if sweep is not None:
        result["ratio_sweep"] = sweep
        result["ratio_sweep_note"] = sweep_note
    print(json.dumps(result))


def cpu_baseline(cfg, inp, bm):
    """The oracle as it stands (numpy fp64), on a bounded sample of the same workload."""
    from oracle import lasnet_oracle as O
    from paper_2210_06223_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    f = lambda k: (synth.bf16_bits_to_f32(inp.dev[k]) if inp.dev[k].dtype == np.uint16 else inp.dev[k])
    wts = [f(k).astype(np.float64) for k in ("W1", "b1", "W2", "b2", "W3", "b3")]
    Wm = inp.dev["Wm"].astype(np.float64)

    def run(n):
        x = f("x")[:n].astype(np.float64)
        t0 = time.perf_counter()
        mask, idx, cnt, _ = O.masker(x, Wm, bm, cfg.S, 0.0)
        O.sparse_bottleneck(x, mask, cfg.S, *wts)
        return time.perf_counter() - t0

    n = min(cfg.N, 2)
    t = run(n)                                   # also warms the BLAS threads
    n = int(max(1, min(cfg.N, n * 10.0 / max(t, 1e-3))))   # aim at ~10 s of CPU work
    t = run(n)
    return {"value": n / t, "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d of %d images of the same workload, numpy fp64 dense block then mask, %.2f s" % (n, cfg.N, t)}


if __name__ == "__main__":
    main()
