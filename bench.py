#!/usr/bin/env python3
"""Benchmark of the LASNet sparse-bottleneck hot path on one MI355X.

One "step" = the whole path over one synthetic batch that is already resident in HBM:
lasnet_masker_ex (pool -> logit -> threshold -> index list, inactive cells passed through to
out) followed by lasnet_sparse_bottleneck_ex (gather + conv1 / conv3x3 / conv3 + scatter-add
on the active cells), with the active-patch count staying on the device.  Every element of
out is written in every step.  Default workload: ResNet-101 stage-3
bottleneck, 14x14x1024, mid 256, S=2, batch 128, bf16, masker calibrated to r = 0.5.

Prints ONE JSON line: whole-job images/s, plus
  roofline      the block's dominant kernel against the bf16 MFMA peak on ACTIVE FLOPs
                (r * N * H*W * 34*M^2; halo recompute is never credited) or against the HBM peak
                on algorithmic bytes, whichever bounds it; duration measured here with events on
                the launch stream; the fractions are also given against the peaks this GPU sustains
                in two microbenchmarks (register-only MFMA loop, stream copy);
  ratio_sweeps  latency of the block against the activation ratio (0.1 .. 1, per-image ratios
                Beta-distributed, iid cells and one blob per image) for the workload and for the
                28x28x512 block the sweep is defined on, against the dense block;
  cpu_baseline  the numpy fp64 oracle timed on this machine's host cores on a bounded sample.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
SWEEP_RATIOS = (0.1, 0.25, 0.5, 0.75, 1.0)


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
    ap.add_argument("--no-dense", action="store_true",
                    help="skip every dense-baseline leg (profiling runs: where the dense block runs on the sparse "
                         "block's own kernels, a kernel trace then holds the sparse launches only)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the latency-against-ratio sweeps")
    ap.add_argument("--schedule", choices=("auto", "fused", "tiled"), default="auto",
                    help="force the one-kernel or the three-kernel schedule where the shape has both")
    ap.add_argument("--granularity", action="store_true",
                    help="also time the path at every patch size S that divides H and has a matrix-core kernel "
                         "(the latency-ratio-against-S curve of Sec. 4.2 on this GPU)")
    ap.add_argument("--chain", action="store_true",
                    help="instead: the 29 sparse blocks of a ResNet-101 body as a chain (see paper_2210_06223_amd/chain.py)")
    return ap.parse_args()


def source_signature():
    """sha1 over the kernel sources: a stored counter profile belongs to the build it was taken from."""
    h = hashlib.sha1()
    for f in sorted(glob.glob(os.path.join(ROOT, "paper_2210_06223_amd", "csrc", "*"))):
        h.update(open(f, "rb").read())
    return h.hexdigest()[:16]


def stored_traffic(workload, schedule):
    """HBM-side bytes per launch of the block's kernels from the rocprofv3 counter summary under profiles/
    (a line `TRAFFIC_BYTES_PER_LAUNCH <schedule> <bytes> sources <sha>`); None if there is none or if the
    kernel sources have changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic_pmc.txt" % workload)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        m = re.match(r"TRAFFIC_BYTES_PER_LAUNCH\s+(\w+)\s+(\d+)\s+sources\s+(\w+)", line.strip())
        if m and m.group(1) == schedule:
            rel = os.path.relpath(path, ROOT)
            if m.group(3) != source_signature():
                return None, rel + " (stale: kernel sources changed since it was taken)"
            return int(m.group(2)), rel
    return None, None


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
    from paper_2210_06223_amd import build as _build
    if not os.path.exists(_build.LIB):            # a tree that was never built: build it, then load it
        _build.build_all(verbose=False)
    B.lib()  # fail loudly if the library cannot be loaded
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.chain:
        from paper_2210_06223_amd import chain
        print(json.dumps(chain.bench_chain(steps=min(args.steps, 20), warmup=min(args.warmup, 3))))
        return

    forced = {"auto": 0, "fused": B.LASNET_FORCE_FUSED, "tiled": B.LASNET_FORCE_TILED}[args.schedule]

    # ------------------------------------------------------------------ timing helpers
    def timed(fn, reps):
        """Per-call durations from one event pair per call: mean / median / p10 / p90 in ms."""
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

    # ------------------------------------------------------------------ what this GPU sustains
    sink = torch.zeros(4096, dtype=torch.float32, device=dev)
    flops_box = [0.0]

    def mfma_loop(i):
        flops_box[0] = B.lasnet_microbench_mfma(2000, sink)

    mfma_ms = timed_loop(mfma_loop, 10)
    sustained_tflops = flops_box[0] / (mfma_ms * 1e-3) / 1e12
    cp_src = torch.empty(512 * 1024 * 1024, dtype=torch.uint8, device=dev)     # 2 x 512 MiB >> the 256 MB cache
    cp_dst = torch.empty_like(cp_src)
    copy_ms = timed_loop(lambda i: B.lasnet_microbench_copy(cp_src, cp_dst), 10)
    sustained_gbs = 2 * cp_src.numel() / (copy_ms * 1e-3) / 1e9
    del cp_src, cp_dst
    # every CU reading the same 2.25 MiB (the size of the 14x14x1024 block's weights) from L2, as the block kernels do
    ws_buf = torch.zeros(18 * 128 * 1024, dtype=torch.uint8, device=dev)
    ws_box = [0.0]

    def ws_loop(i):
        ws_box[0] = B.lasnet_microbench_weight_stream(ws_buf, 20, sink)

    ws_ms = timed_loop(ws_loop, 10)
    ws_gbs = ws_box[0] / (ws_ms * 1e-3) / 1e9
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    achievable = {"mfma_bf16_tflops": sustained_tflops, "mfma_frac_of_nominal": sustained_tflops / PEAK_BF16_TFLOPS,
                  "stream_copy_gbs": sustained_gbs, "copy_frac_of_nominal": sustained_gbs / PEAK_HBM_GBS,
                  "weight_stream_gbs": ws_gbs, "weight_stream_gbs_per_cu": ws_gbs / n_cu,
                  "weight_stream_us_per_pass_of_2.25MiB": ws_buf.numel() / (ws_gbs / n_cu * 1e9) * 1e6,
                  "note": "register-only v_mfma_f32_16x16x32_bf16 loop on every SIMD (4 waves each, 16 independent "
                          "accumulators); out = in over 512 MiB with 16 bytes per lane (read + written bytes counted); "
                          "one 8-wave workgroup per CU, all reading the same 2.25 MiB from L2 in 1 KiB wave-wide pieces, "
                          "16 loads per lane in flight (what a CU's weight stream can reach when every CU streams)"}

    # ------------------------------------------------------------------ one workload
    def load(cfg):
        inp = synth.make_block_inputs(cfg, want_f64=False)

        def to_dev(k, v):
            if cfg.dtype == "bf16" and k in ("x", "W1", "W2", "W3"):
                return torch.from_numpy(v.view(np.int16)).view(torch.bfloat16).to(dev)
            return torch.from_numpy(v).to(dev)

        return inp, {k: to_dev(k, v) for k, v in inp.dev.items()}

    def ratio_sweep(cfg, d, xs, outs, packed, dense_ms, forced=0):
        """Block latency against the activation ratio: index lists fed directly (per-image ratios
        Beta-distributed around the mean), prepacked weights, identity pass-through not included (it lives
        in the masker call), against the dense block through the same entry."""
        pts = []
        P, S = cfg.P, cfg.S
        for r in SWEEP_RATIOS:
            for structure in ("iid", "blob"):
                il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, r, seed=cfg.seed, structure=structure)
                idx_r = torch.zeros((P,), dtype=torch.int32, device=dev)
                idx_r[: len(il)] = torch.from_numpy(il).to(dev)
                cnt_r = torch.tensor([len(il)], dtype=torch.int32, device=dev)
                t = sorted(timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
                    xs[i % len(xs)], idx_r, cnt_r, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[i % len(xs)],
                    flags=B.LASNET_SKIP_IDENTITY | forced), 100) for _ in range(3))[1]
                try:                 # the library's latency predictor (fitted constants, Sec. 3.3 / App. A in this chip's terms)
                    from paper_2210_06223_amd import latency_model as LM
                    sch = "tiled" if forced == B.LASNET_FORCE_TILED else "fused" if forced == B.LASNET_FORCE_FUSED else "auto"
                    pred = LM.predict_us(il, cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, S, sch) * 1e-3
                except Exception:
                    pred = None
                pts.append({"r_mean": r, "structure": structure, "active": len(il), "r": len(il) / P,
                            "block_ms": t, "latency_ratio_vs_dense": t / dense_ms, "predicted_ms": pred})
        # how far the curve is from affine in r: worst deviation of a point from the line through the end points
        for structure in ("iid", "blob"):
            q = [p for p in pts if p["structure"] == structure]
            (r0, t0), (r1, t1) = (q[0]["r"], q[0]["block_ms"]), (q[-1]["r"], q[-1]["block_ms"])
            dev_max = max(abs(p["block_ms"] - (t0 + (t1 - t0) * (p["r"] - r0) / (r1 - r0))) / p["block_ms"] for p in q)
            for p in q:
                p["max_deviation_from_affine"] = dev_max
        return pts

    cfg = synth.CONFIGS[args.workload]
    if args.ratio is not None:
        cfg = cfg.with_(r=args.ratio)
    inp, d = load(cfg)
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
    flags_step = B.LASNET_SKIP_IDENTITY | forced

    def step(i):
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker_ex(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count, pass_out=out)
        B.lasnet_sparse_bottleneck(x, idx, count, S, *w, out=out, flags=flags_step)

    def step_separate_copy(i):       # the two spec calls as they are: identity copy inside the block call
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count)
        B.lasnet_sparse_bottleneck(x, idx, count, S, *w, out=out, flags=forced)

    fast = cfg.dtype == "bf16" and B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, S) == 1
    packed = B.lasnet_pack_weights(S, d["W1"], d["W2"], d["W3"]) if fast else None   # once, like BN folding
    ws_bytes = B.lasnet_workspace_bytes(d["x"], cfg.M, S) if fast else 0
    workspace = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None

    def block_packed(i, idx_=None, cnt_=None, flags=None):
        B.lasnet_sparse_bottleneck_packed(xs[i % nbuf], idx if idx_ is None else idx_, count if cnt_ is None else cnt_,
                                          S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf],
                                          flags=flags_step if flags is None else flags)

    def step_packed(i):
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker_ex(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count, pass_out=out)
        block_packed(i)

    def step_planned(i):             # prepacked weights, caller's workspace, the masker's mask handed on
        x, out = xs[i % nbuf], outs[i % nbuf]
        B.lasnet_masker_ex(x, d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count, pass_out=out)
        B.lasnet_sparse_bottleneck_planned(x, idx, count, mask, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out,
                                           workspace, flags=flags_step)

    def run_steps(fn):
        for i in range(args.warmup):
            fn(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            fn(i)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    dt_packed = run_steps(step_packed) if fast else None
    dt_planned = run_steps(step_planned) if fast else None
    dt_separate = run_steps(step_separate_copy)
    dt = run_steps(step)
    ms_per_step = dt / args.steps * 1e3
    images_per_s = cfg.N * args.steps / dt
    n_active = int(count.item())
    reps = max(20, min(args.steps, 200))
    step_dist = timed(step, reps)    # per-step distribution (event pair per step, on the launch stream)

    # ---- the block alone: same launch as inside the step, identity copy skipped (outs already hold x) ----
    if fast:
        fused_t = timed(block_packed, reps)
        fused_loop_ms = timed_loop(block_packed, reps)
        fused_warm_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[0], idx, count, S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=outs[0], flags=flags_step), reps)
    else:
        blk = lambda i: B.lasnet_sparse_bottleneck(xs[i % nbuf], idx, count, S, *w, out=outs[i % nbuf], flags=flags_step)
        fused_t = timed(blk, reps)
        fused_loop_ms = timed_loop(blk, reps)
        fused_warm_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck(xs[0], idx, count, S, *w, out=outs[0],
                                                                        flags=flags_step), reps)
    block_t = timed(lambda i: B.lasnet_sparse_bottleneck(xs[i % nbuf], idx, count, S, *w, out=outs[i % nbuf], flags=forced), reps)
    masker_t = timed(lambda i: B.lasnet_masker(xs[i % nbuf], d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count), reps)
    masker_ex_t = timed(lambda i: B.lasnet_masker_ex(xs[i % nbuf], d["Wm"], bm, S, 0.0, mask=mask, idx=idx, count=count,
                                                     pass_out=outs[i % nbuf]), reps)
    dense_t = None if args.no_dense else timed(
        lambda i: B.lasnet_dense_bottleneck(xs[i % nbuf], *w, out=outs[i % nbuf], flags=forced), reps)
    # the dense block through the prepacked entry: every cell active (idx = NULL) on the tile side that
    # lasnet_dense_bottleneck picks (the largest built S that divides H and W)
    dense_packed_ms = None
    if fast and not args.no_dense:
        S_dense = max(s_ for s_ in range(1, 17) if cfg.H % s_ == 0 and cfg.W % s_ == 0
                      and B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, s_) == 1)
        packed_dense = B.lasnet_pack_weights(S_dense, d["W1"], d["W2"], d["W3"])
        dense_packed_ms = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
            xs[i % nbuf], None, None, S_dense, cfg.M, packed_dense, d["b1"], d["b2"], d["b3"], out=outs[i % nbuf],
            flags=forced), reps)

    torch_dense = None
    if not args.no_torch_dense and not args.no_dense and cfg.dtype == "bf16":
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
    fused_s = fused_loop_ms * 1e-3             # average duration of the block over `reps` back-to-back calls
    achieved_tflops = active_flops / fused_s / 1e12
    esize = 2 if cfg.dtype == "bf16" else 4
    x_bytes = cfg.N * cfg.H * cfg.W * cfg.C * esize
    # Algorithmic bytes of one launch of the block: every pixel some active patch's (S+2)x(S+2)
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
    tiled = fast and ws_bytes > 0 and args.schedule != "fused" and (args.schedule == "tiled" or (cfg.C, cfg.M) == (2048, 512))
    # The tiled schedule's own minimum adds what its three kernels hand on through memory: y1 of every needed
    # pixel and y2 of every active pixel written once and read once, and the residual read again by the third.
    alg_bytes_path = alg_bytes
    if tiled:
        alg_bytes += (2 * int(pix_need.sum()) + 2 * int(pix_act.sum())) * cfg.M * esize + int(pix_act.sum()) * cfg.C * esize
    achieved_gbs = alg_bytes / fused_s / 1e9
    schedule = "generic" if not fast else "tiled" if tiled else "stream" if (cfg.C, cfg.M, S) == (256, 64, 8) else "fused"
    kernel_name = {"generic": "bneck_generic_kernel", "stream": "stream_bneck_kernel", "fused": "fused_bneck_kernel",
                   "tiled": "tiled_conv1_kernel + tiled_conv2_kernel + tiled_conv3_kernel (one block = three launches; "
                            "per-kernel durations: profiles/)"}[schedule]
    # the bound is whichever ideal time is longer: active FLOPs at the MFMA peak or these bytes at the HBM peak
    hbm_bound = alg_bytes / (PEAK_HBM_GBS * 1e9) > active_flops / (PEAK_BF16_TFLOPS * 1e12)
    dense_best = None if args.no_dense else dense_t["mean_ms"] if dense_packed_ms is None else dense_packed_ms
    dense_best_which = "lasnet_dense_bottleneck" if dense_packed_ms is None else "own dense block, prepacked"
    if torch_dense and "mean_ms" in torch_dense and torch_dense["mean_ms"] < dense_best:
        dense_best, dense_best_which = torch_dense["mean_ms"], "torch/MIOpen conv stack"
    traffic, traffic_source = stored_traffic(cfg.name, schedule) if args.ratio is None else (None, None)

    sweeps = None
    if not args.no_sweep and not args.no_dense and fast:
        sweeps = {cfg.name: ratio_sweep(cfg, d, xs, outs, packed, dense_packed_ms, forced)}
        sweeps_dense = {cfg.name: dense_packed_ms}
        if cfg.name != "stage2_b128" and args.ratio is None and args.workload == "stage3_b128":
            # the 28x28x512 block on which the ratio sweep is defined
            del xs[1:], outs[1:]
            cfg2 = synth.CONFIGS["stage2_b128"]
            inp2, d2 = load(cfg2)
            xs2 = [d2["x"]] + [d2["x"].clone() for _ in range(2)]
            outs2 = [torch.empty_like(d2["x"]) for _ in range(3)]
            packed2 = B.lasnet_pack_weights(cfg2.S, d2["W1"], d2["W2"], d2["W3"])
            packed2d = B.lasnet_pack_weights(7, d2["W1"], d2["W2"], d2["W3"])
            dense2 = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
                xs2[i % 3], None, None, 7, cfg2.M, packed2d, d2["b1"], d2["b2"], d2["b3"], out=outs2[i % 3]), 100)
            sweeps[cfg2.name] = ratio_sweep(cfg2, d2, xs2, outs2, packed2, dense2)
            sweeps_dense[cfg2.name] = dense2
            del xs2, outs2, d2, inp2

    gran = None
    if args.granularity and not args.no_dense and fast:
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
            nb = len(xs)

            def step_g(i):
                B.lasnet_masker_ex(xs[i % nb], d["Wm"], bm_g, S_g, 0.0, mask=mask_g, idx=idx_g, count=cnt_g,
                                   pass_out=outs[i % nb])
                B.lasnet_sparse_bottleneck_packed(xs[i % nb], idx_g, cnt_g, S_g, cfg.M, packed_g, d["b1"], d["b2"],
                                                  d["b3"], out=outs[i % nb], flags=flags_step)

            t_step = timed_loop(step_g, 50)
            t_block = timed_loop(lambda i: B.lasnet_sparse_bottleneck_packed(
                xs[i % nb], idx_g, cnt_g, S_g, cfg.M, packed_g, d["b1"], d["b2"], d["b3"], out=outs[i % nb],
                flags=flags_step), 50)
            gran.append({"S": S_g, "cells": Pg, "active": int(cnt_g.item()), "step_ms": t_step, "block_ms": t_block,
                         "latency_ratio_vs_dense_block": t_block / dense_ms,
                         "latency_ratio_step_vs_dense_block": t_step / dense_ms})

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(cfg, inp, bm)

    frac_mfma = achieved_tflops / PEAK_BF16_TFLOPS
    frac_hbm = achieved_gbs / PEAK_HBM_GBS
    result = {
        "metric": "sparse bottleneck images/s at r=%.2g (masker + index list + identity pass-through + block)" % cfg.r,
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
                   "buffers_rotated": nbuf, "masker_margin": margin, "schedule": schedule},
        "step_ms": step_dist,
        "active_tflops_whole_step": active_flops / (ms_per_step * 1e-3) / 1e12,
        "prepacked_weights": None if dt_packed is None else {
            "ms_per_step": dt_packed / args.steps * 1e3, "images_per_s": cfg.N * args.steps / dt_packed,
            "note": "same step through lasnet_sparse_bottleneck_packed (weights repacked once, outside the loop)"},
        "planned": None if dt_planned is None else {
            "ms_per_step": dt_planned / args.steps * 1e3, "images_per_s": cfg.N * args.steps / dt_planned,
            "note": "same step through lasnet_sparse_bottleneck_planned (prepacked weights, caller's workspace, "
                    "the masker's byte mask handed on)"},
        "separate_identity_copy": {
            "ms_per_step": dt_separate / args.steps * 1e3, "images_per_s": cfg.N * args.steps / dt_separate,
            "note": "lasnet_masker + lasnet_sparse_bottleneck: the block call copies x to out before its kernels"},
        "speedup_vs_dense": None if dense_best is None else dense_best / (fused_loop_ms if fast else block_t["mean_ms"]),
        "speedup_vs_dense_note": None if dense_best is None else
        "dense block (%s, the fastest of the library's own and torch/MIOpen's, %.4f ms) / sparse "
        "block at this r, both without the identity pass-through, which lives in the masker call"
        % (dense_best_which, dense_best),
        "kernels_ms": {"masker+compaction": masker_t, "masker+identity+compaction": masker_ex_t,
                       "pack+copy+block": block_t, "block": fused_t,
                       "dense_own": dense_t, "dense_own_prepacked_loop_ms": dense_packed_ms,
                       "block_loop_ms": fused_loop_ms, "block_warm_loop_ms": fused_warm_ms, "dense_torch_miopen": torch_dense},
        "hbm_floor_ms": 2 * x_bytes / (PEAK_HBM_GBS * 1e9) * 1e3,
        "roofline": {"bound": "hbm" if hbm_bound else "mfma", "kernel": kernel_name,
                     "achieved": achieved_gbs if hbm_bound else achieved_tflops,
                     "peak": PEAK_HBM_GBS if hbm_bound else PEAK_BF16_TFLOPS,
                     "unit": "GB/s" if hbm_bound else "TFLOP/s",
                     "frac": frac_hbm if hbm_bound else frac_mfma,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "active_flops_per_launch": active_flops, "algorithmic_bytes_per_launch": alg_bytes,
                     "algorithmic_bytes_of_the_path": alg_bytes_path,
                     "frac_of_mfma_peak": frac_mfma, "frac_of_hbm_peak": frac_hbm,
                     "frac_of_sustained_mfma": achieved_tflops / sustained_tflops,
                     "frac_of_sustained_copy": achieved_gbs / sustained_gbs,
                     "avg_launch_ms": fused_loop_ms,
                     "avg_launch_ms_single_event_pairs": fused_t["mean_ms"], "launches_timed": reps},
        "achievable": achievable,
        "cpu_baseline": cpu,
        "paper_context": "context only, other hardware and precision, not a target: the paper reports ResNet-101 ImageNet "
                         "latency reduced by 36 % on a Tesla V100 and 46 % on a Jetson TX2 at a FLOPs target of 0.4 "
                         "without accuracy loss (FP32, batch 1, Sec. 1 / 4.3)",
    }
    if gran is not None:
        result["granularity_sweep"] = gran
        result["granularity_sweep_note"] = ("r = %.2f at every S (masker bias recalibrated per S); prepacked weights; "
                                            "dense block %.4f ms; mean over 50 back-to-back launches" % (cfg.r, dense_packed_ms))
    if sweeps is not None:
        result["ratio_sweeps"] = sweeps
        result["ratio_sweeps_note"] = {"dense_ms": sweeps_dense,
                                       "timing": "median of 3 loops of 100 back-to-back launches between two events; prepacked weights; "
                                                 "max_deviation_from_affine: worst relative distance of a point from the "
                                                 "straight line through the r=0.1 and r=1 points of its curve"}
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
    per_image = t / n
    n = int(max(1, min(cfg.N, 10.0 / max(per_image, 1e-6))))   # aim at ~10 s of CPU work:
    passes = int(max(1, min(40, 10.0 / max(per_image * n, 1e-3))))   # a slice of the batch, or the whole batch several times
    t = sum(run(n) for _ in range(passes))
    return {"value": n * passes / t, "unit": "images/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d of %d images of the same workload, %d pass(es), numpy fp64 dense block then mask, %.2f s"
                      % (n, cfg.N, passes, t)}


if __name__ == "__main__":
    main()
