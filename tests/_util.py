"""Helpers shared by the GPU parity tests: host<->device marshalling and the tolerance rule."""
import numpy as np
import torch

from oracle import lasnet_oracle as O
from paper_2210_06223_amd import synth

RTOL = {"f32": 1e-4, "bf16": 2e-2}     # spec tolerances: relative, fp32 / bf16 with fp32 accumulate


def to_dev(arr: np.ndarray, dtype: str, is_feature: bool) -> torch.Tensor:
    """numpy storage array -> device tensor (uint16 bit patterns become bfloat16)."""
    if dtype == "bf16" and is_feature:
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(np.ascontiguousarray(arr)).cuda()


def dev_inputs(inp: synth.BlockInputs):
    dt = inp.cfg.dtype
    d = {k: to_dev(v, dt, k in ("x", "W1", "W2", "W3")) for k, v in inp.dev.items()}
    return d


def weights(d):
    return (d["W1"], d["b1"], d["W2"], d["b2"], d["W3"], d["b3"])


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw bit patterns of a device tensor, for bit-exact comparisons."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.view(torch.int32).numpy().view(np.uint32)
    return t.numpy()


def calibrate(inp: synth.BlockInputs, k: int, thr: float = 0.0):
    """Masker bias for exactly k active cells, from the ORACLE's bias-free logits."""
    cfg = inp.cfg
    logits0 = O.masker_logits(inp.f64["x"], inp.f64["Wm"], 0.0, cfg.S)
    bm, margin = synth.bias_for_count(logits0, k, thr)
    # fp64 summation noise is ~1e-16 * sum|terms|; demand nine orders of magnitude more
    scale = float(np.abs(inp.f64["Wm"]).sum() * inp.f64["x"].max())
    assert margin > 1e-9 * scale, "masker margin too small for an order-independent mask; reseed"
    return bm


def assert_block_close(got: torch.Tensor, ref: np.ndarray, x: torch.Tensor, up_mask: np.ndarray,
                       dtype: str, what: str = ""):
    """Active positions within tolerance, inactive positions bit-identical to x.

    Tolerance (derived in the design notes): |got - ref| <= rtol*|ref| + rtol*rms(ref_active),
    max|got - ref| <= rtol * max|ref|, and the relative L2 error over the active positions <= rtol.
    """
    rtol = RTOL[dtype]
    g = to_f64(got)
    assert np.isfinite(g).all(), what + ": non-finite output"
    act = up_mask.astype(bool)
    if (~act).any():
        gb, xb = bits(got), bits(x)
        assert np.array_equal(gb[~act], xb[~act]), what + ": inactive positions differ from x"
    if act.any():
        ga, ra = g[act], ref[act]
        rms = float(np.sqrt(np.mean(ra * ra)))
        err = np.abs(ga - ra)
        bound = rtol * np.abs(ra) + rtol * rms
        worst = float((err / bound).max())
        assert worst <= 1.0, "%s: per-element error %.3g x bound (max abs err %.3g, rms %.3g)" % (
            what, worst, float(err.max()), rms)
        assert float(err.max()) <= rtol * float(np.abs(ra).max()), what + ": max-norm error"
        rel_l2 = float(np.sqrt(np.sum(err * err) / max(np.sum(ra * ra), 1e-300)))
        assert rel_l2 <= rtol, "%s: relative L2 error %.3g > %.3g" % (what, rel_l2, rtol)


def list_tensor(entries: np.ndarray, P: int) -> torch.Tensor:
    """An index list in storage of the size the masker writes to: P entries, the unused tail poisoned."""
    t = torch.full((max(int(P), 1),), -7, dtype=torch.int32, device="cuda")
    if len(entries):
        t[: len(entries)] = torch.from_numpy(np.asarray(entries, np.int32)).cuda()
    return t
