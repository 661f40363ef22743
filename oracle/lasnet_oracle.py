"""CPU oracle for the LASNet coarse-grained sparse bottleneck block.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this; it is
used by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg.
It shares no code with the HIP path and never sees a value the HIP path made.

The fast path skips work, it does not approximate, so the oracle is the plain
definition written out in numpy fp64: compute the whole dense block, then apply
the upsampled patch mask to the block's residual branch,

    out = x + up_S(M_coarse) * F(x)                       (Sec. 3.1, Sec. 3.2)

with no gather, no index list inside the block and no tiling.  Layout is NHWC,
weights are [out][in] (W2: [out][ky][kx][in]) with BN already folded in
(Sec. 3.4, first paragraph).

Readings of passages the paper leaves open (all restated in the design notes):
  * the masker's pooling (Sec. 3.2 does not say which) = average pool, kernel = stride = S.
  * inference decision = strict `logit > thr` (App. B.1 equation uses `>`;
    thr generalises its 0); a tie is inactive.
  * the 3x3 conv zero-pads conv1's OUTPUT (as the dense ResNet block does).
  * no ReLU after the residual add unless post_relu=True, which then acts on
    active patches only (inactive patches stay bit-identical to x).
  * index list = ascending flat cell ids n*G*GW + gy*GW + gx (App. B.1 (2)).

Pins: tests/test_oracle_pins.py (closed forms, torch conv2d/avg_pool2d in fp64,
pure-python per-patch brute force, impulse-response geometry, invariants).
"""
from __future__ import annotations

import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


# --------------------------------------------------------------------------- masker
def masker_logits(x, Wm, bm, S):
    """logit[n,gy,gx] = bm + sum_c Wm[c] * mean_{SxS patch}(x)[n,gy,gx,c]   (Sec. 3.2:
    pooling layer then 1x1 convolution; App. B.1: one output channel suffices)."""
    x = _f64(x)
    N, H, W, C = x.shape
    if H % S or W % S:
        raise ValueError("S must divide H and W (Sec. 3.2 lists divisors only)")
    G, GW = H // S, W // S
    pooled = x.reshape(N, G, S, GW, S, C).sum(axis=(2, 4)) / float(S * S)
    return float(bm) + pooled @ _f64(Wm)


def index_list(mask):
    """Ascending flat ids of active cells, and their number (App. B.1 (2): the masker
    emits indices of activated patches instead of a sparse mask)."""
    flat = np.asarray(mask).reshape(-1)
    idx = np.flatnonzero(flat != 0).astype(np.int32)
    return idx, int(idx.size)


def masker(x, Wm, bm, S, thr=0.0):
    """Returns (mask uint8 [N,G,GW], idx int32 [count], count, logits fp64)."""
    logits = masker_logits(x, Wm, bm, S)
    mask = (logits > float(thr)).astype(np.uint8)      # strict, App. B.1 equation
    idx, count = index_list(mask)
    return mask, idx, count, logits


# --------------------------------------------------------------------------- block
def residual_branch(x, W1, b1, W2, b2, W3, b3):
    """F(x) of the ResNet bottleneck with folded BN: 1x1+ReLU, 3x3+ReLU, 1x1 (Sec. 3.2,
    Sec. 3.4).  Dense, at every pixel.  Returns (f, y1, y2)."""
    x = _f64(x)
    W1, W2, W3 = _f64(W1), _f64(W2), _f64(W3)
    N, H, W, C = x.shape
    M = W1.shape[0]
    assert W1.shape == (M, C) and W2.shape == (M, 3, 3, M) and W3.shape == (C, M)
    y1 = np.maximum(x @ W1.T + _f64(b1), 0.0)                        # [N,H,W,M]
    y1p = np.zeros((N, H + 2, W + 2, M))
    y1p[:, 1:H + 1, 1:W + 1, :] = y1                                 # zero padding of y1
    acc = np.zeros((N, H, W, M))
    for ky in range(3):                                              # cross-correlation
        for kx in range(3):
            acc += y1p[:, ky:ky + H, kx:kx + W, :] @ W2[:, ky, kx, :].T
    y2 = np.maximum(acc + _f64(b2), 0.0)
    f = y2 @ W3.T + _f64(b3)                                         # no ReLU before the add
    return f, y1, y2


def upsample_mask(mask, S):
    """Nearest upsample of the coarse mask to H x W (Sec. 3.2)."""
    m = np.asarray(mask)
    return np.repeat(np.repeat(m, S, axis=1), S, axis=2)


def masked_output(x, f, mask, S, post_relu=False):
    """out = x + up_S(mask) * f for a residual branch f = F(x) computed beforehand (F does not
    depend on the mask, so tests that try many masks on one input compute it once)."""
    x = _f64(x)
    up = upsample_mask(mask, S).astype(bool)[..., None]
    y = x + f
    if post_relu:
        y = np.maximum(y, 0.0)
    return np.where(up, y, x)


def sparse_bottleneck(x, mask, S, W1, b1, W2, b2, W3, b3, post_relu=False):
    """out = x + up_S(mask) * F(x): unselected regions keep the input (Sec. 3.1)."""
    x = _f64(x)
    f, _, _ = residual_branch(x, W1, b1, W2, b2, W3, b3)
    return masked_output(x, f, mask, S, post_relu)


def dense_bottleneck(x, W1, b1, W2, b2, W3, b3, post_relu=False):
    """The static block: every position computed (activation rate 1)."""
    x = _f64(x)
    f, _, _ = residual_branch(x, W1, b1, W2, b2, W3, b3)
    y = x + f
    return np.maximum(y, 0.0) if post_relu else y


def block_flops(H, W, C, M, r=1.0):
    """FLOPs (2 per multiply-add) of one block at activation rate r (Sec. 3.5: block
    FLOPs follow from r): conv1 2CM + conv2 18M^2 + conv3 2MC per computed pixel."""
    return r * H * W * (2 * C * M + 18 * M * M + 2 * M * C)
