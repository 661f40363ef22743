"""Seeded synthetic inputs for the LASNet sparse-bottleneck path.

This module only draws random tensors with the shapes, value distributions and
mask structure of the paper's ResNet-101 workloads (Sec. 3.2: S x S patches on
56/28/14/7-sized features; Sec. 4: FLOPs targets t in {0.4..0.7}).  It holds
none of the method's arithmetic: no pooling, no convolution, no compaction.
Both the CPU oracle's tests and the HIP path's harness draw from here so that
they see bit-identical inputs.

Recipe (numpy PCG64, one child stream per tensor in the fixed order
x, W1, s1, b1, W2, s2, b2, W3, s3, b3, Wm):
  x   = ReLU(N(0,1))                       [N,H,W,C]   (block inputs follow a ReLU)
  W1  = N(0, 2/C)      * s1[m]             [M,C]       He-normal, BN scale folded in
  W2  = N(0, 2/(9M))   * s2[o]             [M,3,3,M]   (out, ky, kx, in)
  W3  = N(0, 2/M)      * s3[c]             [C,M]
  s*  = N(1, 0.1),  b* = N(0, 0.1)         folded BN scale / bias (fp32)
  Wm  = N(0, 0.02)                         [C]         masker 1x1 conv (fp32)
For dtype "bf16", x and W1..W3 are rounded once to bfloat16 (nearest-even) on
the host; the fp64 views handed to the oracle hold exactly those rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

__all__ = [
    "BlockConfig", "CONFIGS", "BlockInputs", "make_block_inputs",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "bias_for_count",
    "make_index_list",
]


@dataclass(frozen=True)
class BlockConfig:
    """Shape of one bottleneck workload (names follow the paper: H, W, C, S, r)."""
    name: str
    N: int
    H: int
    W: int
    C: int          # block input / output channels
    M: int          # bottleneck (mid) channels
    S: int          # spatial granularity (patch side)
    dtype: str      # "f32" | "bf16"
    r: float        # target activation ratio
    seed: int

    @property
    def G(self) -> int:
        return self.H // self.S

    @property
    def GW(self) -> int:
        return self.W // self.S

    @property
    def P(self) -> int:
        return self.N * self.G * self.GW

    def with_(self, **kw) -> "BlockConfig":
        d = dict(self.__dict__)
        d.update(kw)
        return BlockConfig(**d)


CONFIGS: Dict[str, BlockConfig] = {
    # tiny fp32 correctness case
    "tiny_f32": BlockConfig("tiny_f32", 1, 16, 16, 64, 16, 4, "f32", 0.5, 0),
    # ResNet-101 stage 3 (headline workload at N=128)
    "stage3_b1": BlockConfig("stage3_b1", 1, 14, 14, 1024, 256, 2, "bf16", 0.5, 1),
    "stage3_b128": BlockConfig("stage3_b128", 128, 14, 14, 1024, 256, 2, "bf16", 0.5, 1),
    # ResNet-101 stage 1, memory bound
    "stage1_b64": BlockConfig("stage1_b64", 64, 56, 56, 256, 64, 8, "bf16", 0.4, 2),
    # ResNet-101 stage 2, ratio sweep
    "stage2_b128": BlockConfig("stage2_b128", 128, 28, 28, 512, 128, 4, "bf16", 0.5, 3),
    # ResNet-101 stage 4: 7x7 maps, pixel-level patches (S = 1)
    "stage4_b128": BlockConfig("stage4_b128", 128, 7, 7, 2048, 512, 1, "bf16", 0.5, 4),
}


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class BlockInputs:
    """One block's tensors.

    `dev[...]`: arrays in storage form for the device (fp32, or uint16 bfloat16
    bit patterns for x/W1/W2/W3 when cfg.dtype == "bf16"; biases and Wm fp32).
    `f64[...]`: the same values widened exactly to fp64 for the oracle.
    """
    cfg: BlockConfig
    dev: Dict[str, np.ndarray] = field(default_factory=dict)
    f64: Dict[str, np.ndarray] = field(default_factory=dict)


def make_block_inputs(cfg: BlockConfig, want_f64: bool = True) -> BlockInputs:
    ss = np.random.SeedSequence(cfg.seed)
    names = ["x", "W1", "s1", "b1", "W2", "s2", "b2", "W3", "s3", "b3", "Wm"]
    gens = {n: np.random.Generator(np.random.PCG64(s)) for n, s in zip(names, ss.spawn(len(names)))}
    N, H, W, C, M = cfg.N, cfg.H, cfg.W, cfg.C, cfg.M

    def normal(name, shape, std=1.0, mean=0.0):
        return (gens[name].standard_normal(shape, dtype=np.float32) * np.float32(std)
                + np.float32(mean)).astype(np.float32)

    raw = {}
    raw["x"] = np.maximum(normal("x", (N, H, W, C)), np.float32(0))
    s1 = normal("s1", (M,), 0.1, 1.0)
    s2 = normal("s2", (M,), 0.1, 1.0)
    s3 = normal("s3", (C,), 0.1, 1.0)
    raw["W1"] = normal("W1", (M, C), np.sqrt(2.0 / C)) * s1[:, None]
    raw["W2"] = normal("W2", (M, 3, 3, M), np.sqrt(2.0 / (9 * M))) * s2[:, None, None, None]
    raw["W3"] = normal("W3", (C, M), np.sqrt(2.0 / M)) * s3[:, None]
    raw["b1"] = normal("b1", (M,), 0.1)
    raw["b2"] = normal("b2", (M,), 0.1)
    raw["b3"] = normal("b3", (C,), 0.1)
    raw["Wm"] = normal("Wm", (C,), 0.02)

    out = BlockInputs(cfg)
    for k, v in raw.items():
        v = np.ascontiguousarray(v, dtype=np.float32)
        if cfg.dtype == "bf16" and k in ("x", "W1", "W2", "W3"):
            bits = f32_to_bf16_bits(v)
            out.dev[k] = bits
            if want_f64:
                out.f64[k] = bf16_bits_to_f32(bits).astype(np.float64)
        else:
            out.dev[k] = v
            if want_f64:
                out.f64[k] = v.astype(np.float64)
    return out


def bias_for_count(logits_nobias: np.ndarray, k: int, thr: float = 0.0):
    """Pick the masker bias so that exactly `k` cells have logit > thr.

    `logits_nobias` are fp64 bias-free logits supplied by the caller (this
    module computes none).  The bias puts `thr` midway between the k-th and
    (k+1)-th largest logit, then is rounded to fp32 (the storage type of bm).
    Returns (bm as python float holding an fp32 value, margin) where margin is
    the smallest |logit + bm - thr| -- callers assert it dwarfs fp64 summation
    noise so that every summation order yields the same mask.
    """
    flat = np.sort(np.asarray(logits_nobias, dtype=np.float64).ravel())[::-1]
    P = flat.size
    if not 0 <= k <= P:
        raise ValueError("k out of range")
    if k == 0:
        edge = flat[0] + 1.0
    elif k == P:
        edge = flat[-1] - 1.0
    else:
        edge = 0.5 * (flat[k - 1] + flat[k])
    bm = float(np.float32(thr - edge))
    margin = float(np.min(np.abs(flat + bm - thr)))
    return bm, margin


def make_index_list(N: int, G: int, GW: int, r_mean: float, seed: int,
                    kappa: float = 10.0, structure: str = "iid",
                    order: str = "ascending") -> np.ndarray:
    """Draw an active-patch index list directly (no masker), for ratio sweeps.

    Per-image ratio r_n ~ Beta(kappa*r, kappa*(1-r)) (r_mean == 1 -> all active,
    0 -> none); round(G*GW*r_n) cells per image.  structure "iid": cells chosen
    uniformly; "blob": the cells nearest (Chebyshev, then raster) to a random
    centre -- one contiguous foreground region per image.  Flat id =
    n*G*GW + gy*GW + gx.  order: "ascending" | "shuffled".
    """
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, 0xA11CE])))
    cells = G * GW
    ids = []
    for n in range(N):
        if r_mean >= 1.0:
            k = cells
        elif r_mean <= 0.0:
            k = 0
        else:
            rn = rng.beta(kappa * r_mean, kappa * (1.0 - r_mean))
            k = int(round(cells * rn))
        if structure == "iid":
            sel = rng.choice(cells, size=k, replace=False)
        elif structure == "blob":
            cy, cx = rng.integers(0, G), rng.integers(0, GW)
            gy, gx = np.divmod(np.arange(cells), GW)
            d = np.maximum(np.abs(gy - cy), np.abs(gx - cx)) * cells + np.arange(cells)
            sel = np.argsort(d, kind="stable")[:k]
        else:
            raise ValueError(structure)
        ids.append(np.sort(sel) + n * cells)
    idx = np.concatenate(ids).astype(np.int32) if ids else np.zeros(0, np.int32)
    if order == "shuffled":
        rng.shuffle(idx)
    elif order != "ascending":
        raise ValueError(order)
    return idx


# --------------------------------------------------------------------------- ResNet-101 body
# Stage shapes of the ResNet-101 body on 224x224 inputs: (H = W, C, M, S, sparse blocks).  The first
# block of every stage (projection shortcut; stride 2 from the second stage on) and the stem run
# dense and are not part of the sparse path; S = (8, 4, 2, 1) per stage, the 7x7 stage pixel-level
# (Sec. 4.2, Sec. 4.3).
RESNET101_STAGES = ((56, 256, 64, 8, 2), (28, 512, 128, 4, 3), (14, 1024, 256, 2, 22), (7, 2048, 512, 1, 2))


def make_chain_weights(seed: int = 4, stages=RESNET101_STAGES, w3_scale_mean: float = 0.25):
    """Random-init weights of every SPARSE block of the body, in order, plus each block's target ratio.

    Per block the recipe of make_block_inputs (He-normal, folded BN scale and bias, masker weights), with
    one change: the folded scale of the LAST convolution is N(w3_scale_mean, w3_scale_mean / 10) instead
    of N(1, 0.1) -- in a random-weight chain the residual branch is as large as the identity and the
    variance of the activations would double with every block, which no trained network does.  Target
    activation ratio of each block ~ U(0.3, 0.7).  Returns a list of dicts with fp32 arrays
    (W1 [M,C], b1, W2 [M,3,3,M], b2, W3 [C,M], b3, Wm [C]), 'stage', 'H', 'C', 'M', 'S', 'r'.
    """
    root = np.random.SeedSequence([seed, 0xB0D1])
    blocks = []
    n_blocks = sum(s[4] for s in stages)
    children = root.spawn(n_blocks)
    bi = 0
    for si, (H, C, M, S, nb) in enumerate(stages):
        for _ in range(nb):
            g = np.random.Generator(np.random.PCG64(children[bi]))
            bi += 1

            def normal(shape, std=1.0, mean=0.0):
                return (g.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)

            s1, s2 = normal((M,), 0.1, 1.0), normal((M,), 0.1, 1.0)
            s3 = normal((C,), w3_scale_mean / 10.0, w3_scale_mean)
            blk = {
                "W1": normal((M, C), np.sqrt(2.0 / C)) * s1[:, None],
                "W2": normal((M, 3, 3, M), np.sqrt(2.0 / (9 * M))) * s2[:, None, None, None],
                "W3": normal((C, M), np.sqrt(2.0 / M)) * s3[:, None],
                "b1": normal((M,), 0.1), "b2": normal((M,), 0.1), "b3": normal((C,), 0.1),
                "Wm": normal((C,), 0.02),
                "r": float(g.uniform(0.3, 0.7)),
                "stage": si + 1, "H": H, "C": C, "M": M, "S": S,
            }
            blocks.append(blk)
    return blocks
