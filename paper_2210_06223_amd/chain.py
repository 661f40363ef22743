"""The sparse blocks of a ResNet-101 body as a chain, on one GPU (harness, not part of the library).

224x224x3 synthetic images -> stem -> four stages.  The stem and the first block of every stage
(projection shortcut, stride 2 from the second stage on) are dense and lie outside the sparse path:
they run as PyTorch convolutions here (random weights, bf16, channels-last), only to give the sparse
blocks inputs of the right shapes and statistics.  The other 2 + 3 + 22 + 2 = 29 blocks run through the
library: lasnet_masker_ex (mask, index list, identity pass-through) and lasnet_sparse_bottleneck_packed
with LASNET_POST_RELU, patch sizes S = (8, 4, 2, 1) per stage, each block's masker bias calibrated on
the running activations to the block's target ratio ~ U(0.3, 0.7).
"""
from __future__ import annotations

import time
from typing import Callable, List, Optional

import numpy as np
import torch
import torch.nn.functional as F

from . import binding as B
from . import synth


def _bf16(a: np.ndarray, dev) -> torch.Tensor:
    return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(dev)


class _DenseParts:
    """Stem and the four projection blocks as PyTorch ops on NHWC memory (channels-last convolutions)."""

    def __init__(self, seed: int, dev):
        g = torch.Generator().manual_seed(seed)

        def conv_w(o, i, k):
            w = torch.randn((o, i, k, k), generator=g) * float(np.sqrt(2.0 / (i * k * k)))
            return w.to(dev, torch.bfloat16).contiguous(memory_format=torch.channels_last)

        self.stem = conv_w(64, 3, 7)
        self.proj = []
        cin = 64
        for (H, C, M, S, nb) in synth.RESNET101_STAGES:
            self.proj.append({"w1": conv_w(M, cin, 1), "w2": conv_w(M, M, 3), "w3": conv_w(C, M, 1) * 0.25,
                              "ws": conv_w(C, cin, 1)})
            cin = C

    @staticmethod
    def _nhwc(t_nchw: torch.Tensor) -> torch.Tensor:
        return t_nchw.contiguous(memory_format=torch.channels_last).permute(0, 2, 3, 1)   # [N,H,W,C] view, contiguous

    def run_stem(self, img_nhwc: torch.Tensor) -> torch.Tensor:
        x = F.relu(F.conv2d(img_nhwc.permute(0, 3, 1, 2), self.stem, stride=2, padding=3))
        return F.max_pool2d(x, 3, stride=2, padding=1)                                     # NCHW logical

    def run_proj(self, si: int, x_nchw: torch.Tensor) -> torch.Tensor:
        p = self.proj[si]
        stride = 1 if si == 0 else 2
        y = F.relu(F.conv2d(x_nchw, p["w1"]))
        y = F.relu(F.conv2d(y, p["w2"], stride=stride, padding=1))
        y = F.conv2d(y, p["w3"])
        return self._nhwc(F.relu(y + F.conv2d(x_nchw, p["ws"], stride=stride)))


class SparseChain:
    """Holds the device weights of the 29 sparse blocks and runs the body."""

    def __init__(self, N: int, seed: int = 4, dev="cuda:0"):
        self.N, self.dev = N, torch.device(dev)
        self.blocks = synth.make_chain_weights(seed)
        self.dense = _DenseParts(seed, self.dev)
        rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0x1A6E])))
        self.images = _bf16(rng.standard_normal((N, 224, 224, 3), dtype=np.float32), self.dev)
        self.w = []
        for b in self.blocks:
            d = {k: _bf16(b[k], self.dev) for k in ("W1", "W2", "W3")}
            d.update({k: torch.from_numpy(b[k]).to(self.dev) for k in ("b1", "b2", "b3", "Wm")})
            d["packed"] = B.lasnet_pack_weights(b["S"], d["W1"], d["W2"], d["W3"])
            self.w.append(d)
        self.bm: List[Optional[float]] = [None] * len(self.blocks)
        self.margin: List[float] = [0.0] * len(self.blocks)
        self.bufs = {}
        for (H, C, M, S, nb) in synth.RESNET101_STAGES:
            P = N * (H // S) * (H // S)
            self.bufs[H] = {"pong": [torch.empty((N, H, H, C), dtype=torch.bfloat16, device=self.dev) for _ in range(2)],
                            "mask": torch.empty((N, H // S, H // S), dtype=torch.uint8, device=self.dev),
                            "idx": torch.empty((P,), dtype=torch.int32, device=self.dev),
                            "count": torch.zeros((1,), dtype=torch.int32, device=self.dev)}

    def run(self, tap: Optional[Callable] = None, timers=None) -> torch.Tensor:
        """One pass over the body.  The first pass calibrates every masker bias (host round trips); later
        passes enqueue without synchronising.  tap(block index, x, mask, idx, count, out) is called after
        each sparse block (testing).  timers: dict of lists of (name, event, event) to fill."""
        def mark(name):
            if timers is None:
                return None
            e = torch.cuda.Event(enable_timing=True)
            e.record()
            timers.setdefault("marks", []).append((name, e))

        mark("start")
        x_nchw = self.dense.run_stem(self.images)
        mark("stem")
        bi = 0
        x = None
        for si, (H, C, M, S, nb) in enumerate(synth.RESNET101_STAGES):
            x = self.dense.run_proj(si, x_nchw if si == 0 else x.permute(0, 3, 1, 2))
            mark("proj%d" % (si + 1))
            bufs = self.bufs[H]
            for j in range(nb):
                blk, w = self.blocks[bi], self.w[bi]
                out = bufs["pong"][j % 2]
                if self.bm[bi] is None:
                    logits0 = B.lasnet_masker_logits(x, w["Wm"], 0.0, S).cpu().numpy()
                    self.bm[bi], self.margin[bi] = synth.bias_for_count(logits0, int(round(blk["r"] * logits0.size)))
                B.lasnet_masker_ex(x, w["Wm"], self.bm[bi], S, 0.0, mask=bufs["mask"], idx=bufs["idx"],
                                   count=bufs["count"], pass_out=out)
                B.lasnet_sparse_bottleneck_packed(x, bufs["idx"], bufs["count"], S, M, w["packed"], w["b1"], w["b2"],
                                                  w["b3"], out=out, flags=B.LASNET_SKIP_IDENTITY | B.LASNET_POST_RELU)
                if tap is not None:
                    tap(bi, x, bufs["mask"], bufs["idx"], bufs["count"], out)
                x = out
                bi += 1
            mark("sparse%d" % (si + 1))
        return x


def bench_chain(N: int = 128, steps: int = 10, warmup: int = 2) -> dict:
    ch = SparseChain(N)
    ch.run()                                     # calibration pass
    for _ in range(warmup):
        ch.run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ch.run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    timers = {}
    ch.run(timers=timers)
    torch.cuda.synchronize()
    marks = timers["marks"]
    share = {}
    for (n0, e0), (n1, e1) in zip(marks[:-1], marks[1:]):
        share[n1] = e0.elapsed_time(e1)
    sparse_ms = sum(v for k, v in share.items() if k.startswith("sparse"))
    ratios = [b["r"] for b in ch.blocks]
    return {"metric": "ResNet-101 body images/s (29 sparse blocks through the library; stem and 4 projection blocks "
                      "as PyTorch convolutions)",
            "value": N / dt, "unit": "images/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": dt * 1e3, "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "ResNet-101 body, 224x224x3, batch %d, S=(8,4,2,1), per-block ratio ~U(0.3,0.7) "
                                   "(mean %.3f)" % (N, float(np.mean(ratios)))},
            "ms_by_part": share, "sparse_blocks_ms": sparse_ms, "sparse_blocks_share": sparse_ms / sum(share.values()),
            "sparse_blocks_images_per_s": N / (sparse_ms * 1e-3),
            "min_masker_margin": float(min(ch.margin))}
