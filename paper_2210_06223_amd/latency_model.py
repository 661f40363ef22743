"""Latency predictor for the sparse bottleneck on MI355X: l = G(block shape, S, active-patch list).

The paper guides its design with a predictor that takes the block configuration, the granularity S
and the activation rate and returns a latency for a given device, from a model of that device's
processing elements and memory levels (Sec. 3.3, App. A).  This is the same idea re-parameterised
for this library on this GPU: it replays, on the host, how the kernels cut an index list into
workgroups, batches and 16-row MFMA blocks (pure integer logic, mirrored from the kernels'
configurations), and prices the result with a handful of coefficients per schedule that were fitted
to measured latency-against-ratio sweeps (profiles/ratio_sweeps_mi355x.txt):

  fused / streaming kernels   a workgroup's time = sum over its batches of
                                  a + b * (16-row blocks of conv1) + c * (16-row blocks of conv2/conv3)
                                  (+ d when the batch has more than 4 output blocks: conv3 then takes its rows
                                  in two groups and streams its weights twice)
                              a: what a batch costs whatever it holds (all weights stream through the CU,
                              the window set is built, pipelines fill); b, c: matrix work and activations.
                              Workgroups fill the chip's slots in launch order; latency = t0 + makespan.
  tiled schedule              three launches; latency = F + g1 * max blocks of a conv1 tile
                                  + g2 * max over image groups of (blocks + p per pass) of conv2/conv3.

It is a model of THIS implementation (it predicts what the library will take, e.g. to choose S or a
schedule), not of the hardware in general.  Nothing in the product path calls it.
"""
from __future__ import annotations

import json
import os
from typing import Dict, Iterable, List, Sequence, Tuple

import numpy as np

N_CU = 256

# Integer parameters of the kernels' configurations (mirrors csrc/mfma_stage*.hip and tiled_stages.hip):
# (C, M, S) -> patches per batch, y1 rows per batch, workgroups per CU.
FUSED = {
    (256, 64, 8): dict(kind="stream"),
    (512, 128, 4): dict(kind="fused", PPW=4, R1MAX=112, wg_per_cu=2),
    (1024, 256, 2): dict(kind="fused", PPW=32, R1MAX=160, wg_per_cu=1),
    (2048, 512, 1): dict(kind="fused", PPW=16, R1MAX=96, wg_per_cu=1),
}
TILED = {(1024, 256): dict(IMGS=1, T1ROWS=112, C2ROWS=128, C3ROWS=112), (2048, 512): dict(IMGS=2, T1ROWS=112, C2ROWS=128, C3ROWS=112)}

# Fitted on MI355X (microseconds); see fit() and profiles/ratio_sweeps_mi355x.txt.
COEFFS: Dict[str, Dict[str, float]] = {}


def _cells(idx: np.ndarray, G: int, GW: int):
    n, rem = np.divmod(idx.astype(np.int64), G * GW)
    gy, gx = np.divmod(rem, GW)
    return n, gy, gx


def window_pixels(cells: Iterable[Tuple[int, int, int]], S: int, H: int, W: int) -> set:
    """In-image pixels of the (S+2)x(S+2) windows of the given cells (one entry per distinct pixel)."""
    out = set()
    for n, gy, gx in cells:
        for h in range(max(0, gy * S - 1), min(H, gy * S + S + 1)):
            base = (n * H + h) * W
            for w in range(max(0, gx * S - 1), min(W, gx * S + S + 1)):
                out.add(base + w)
    return out


def simulate_fused(idx: np.ndarray, N: int, H: int, W: int, C: int, M: int, S: int) -> List[List[Tuple[int, int]]]:
    """How fused_bneck_kernel cuts the list: per workgroup (in launch order) its batches as
    (conv1 blocks, conv2/conv3 blocks)."""
    p = FUSED[(C, M, S)]
    PPW, R1MAX = p["PPW"], p["R1MAX"]
    slots = N_CU * p["wg_per_cu"]
    G, GW = H // S, W // S
    nact = len(idx)
    if nact == 0:
        return []
    nt = -(-nact // PPW)
    nt = -(-nt // slots) * slots
    grid = -(-(N * G * GW) // PPW)
    grid = min(-(-grid // slots) * slots, N * G * GW)
    nt = min(nt, grid, nact)
    n, gy, gx = _cells(idx, G, GW)
    cells = list(zip(n.tolist(), gy.tolist(), gx.tolist()))
    wgs = []
    for b in range(nt):
        xcd, jx = b & 7, b >> 3
        first = xcd * (nt >> 3) + min(xcd, nt & 7)
        runs = (nt >> 3) + (1 if xcd < (nt & 7) else 0)
        xb, xe = first * nact // nt, (first + runs) * nact // nt
        len0 = (xe - xb) // runs
        extra = (xe - xb) - len0 * runs
        tb = xb + jx * len0 + min(jx, extra)
        te = tb + len0 + (1 if jx < extra else 0)
        batches = []
        e0 = tb
        while e0 < te:
            npb = min(te - e0, PPW)
            while True:
                U = len(window_pixels(cells[e0:e0 + npb], S, H, W))
                if U <= R1MAX:
                    break
                npb = max(1, min(npb - 1, npb * R1MAX // U))
            batches.append((max(1, -(-U // 16)), -(-(npb * S * S) // 16)))
            e0 += npb
        wgs.append(batches)
    return wgs


def _makespan(times: Sequence[float], slots: int) -> float:
    """Workgroups start in launch order, each on the slot that frees first."""
    if len(times) <= slots:
        return max(times) if len(times) else 0.0
    import heapq
    heap = list(times[:slots])
    heapq.heapify(heap)
    for t in times[slots:]:
        heapq.heappush(heap, heapq.heappop(heap) + t)
    return max(heap)


def features(idx: np.ndarray, N: int, H: int, W: int, C: int, M: int, S: int, schedule: str) -> dict:
    """The integer quantities the coefficients multiply."""
    if schedule == "tiled":
        p = TILED[(C, M)]
        G, GW = H // S, W // S
        act = np.zeros((N, G, GW), bool)
        n, gy, gx = _cells(idx, G, GW)
        act[n, gy, gx] = True
        pix = np.repeat(np.repeat(act, S, 1), S, 2)
        pad = np.pad(pix, ((0, 0), (1, 1), (1, 1)))
        need = np.zeros_like(pix)
        for dy in range(3):
            for dx in range(3):
                need |= pad[:, dy:dy + H, dx:dx + W]
        IMGS = p["IMGS"]
        ng = -(-N // IMGS)
        padn = ng * IMGS - N
        A = np.pad(pix.reshape(N, -1).sum(1), (0, padn)).reshape(ng, IMGS).sum(1)
        gpx = IMGS * H * W
        nt1 = -(-gpx // p["T1ROWS"])
        t1px = -(-gpx // nt1)
        needg = np.pad(need.reshape(N, -1), ((0, padn), (0, 0))).reshape(ng, gpx)
        U = np.array([[needg[g, t * t1px:(t + 1) * t1px].sum() for t in range(nt1)] for g in range(ng)])

        def passes(a, cap):
            a = int(a)
            if a == 0:
                return 0, 0
            npass = -(-a // cap)
            return npass, -(-a // 16)

        c2 = [passes(a, p["C2ROWS"]) for a in A]
        c3 = [passes(a, p["C3ROWS"]) for a in A]
        return dict(nb1=int(np.ceil(U.max() / 16.0)), nb2=max(b for _, b in c2), np2=max(q for q, _ in c2),
                    nb3=max(b for _, b in c3), np3=max(q for q, _ in c3), any=int(len(idx) > 0))
    if FUSED[(C, M, S)]["kind"] == "stream":
        nact = len(idx)
        nt = min(N_CU, nact)
        return dict(maxrun=-(-nact // nt) if nt else 0, any=int(nact > 0))
    return dict(wgs=simulate_fused(idx, N, H, W, C, M, S), slots=N_CU * FUSED[(C, M, S)]["wg_per_cu"])


def _predict(f: dict, k: Dict[str, float], schedule: str, kind: str) -> float:
    if schedule == "tiled":
        if not f["any"]:
            return k["F"]
        return k["F"] + k["g1"] * f["nb1"] + k["g2"] * (f["nb2"] + f["nb3"]) + k["p"] * (f["np2"] + f["np3"] - 2)
    if kind == "stream":
        return k["t0"] + k["c"] * f["maxrun"]
    times = [k["w0"] + sum(k["a"] + k["b"] * b1 + k["c"] * b2 + (k.get("d", 0.0) if b2 > 4 else 0.0) for b1, b2 in wg)
             for wg in f["wgs"]]
    return k["t0"] + _makespan(times, f["slots"])


def key_of(C: int, M: int, S: int, schedule: str) -> str:
    return "%dx%d_S%d_%s" % (C, M, S, schedule)


def predict_us(idx: np.ndarray, N: int, H: int, W: int, C: int, M: int, S: int, schedule: str = "auto",
               coeffs: Dict[str, Dict[str, float]] = None) -> float:
    """Predicted latency of the block (prepacked weights, no identity pass-through) in microseconds."""
    coeffs = COEFFS if coeffs is None else coeffs
    if schedule == "auto":
        schedule = "tiled" if (C, M) == (2048, 512) else "fused"
    kind = "tiled" if schedule == "tiled" else FUSED[(C, M, S)]["kind"]
    k = coeffs[key_of(C, M, S, schedule)]
    return _predict(features(np.asarray(idx), N, H, W, C, M, S, schedule), k, schedule, kind)


def fit(points: List[dict]) -> Dict[str, Dict[str, float]]:
    """Least-squares coefficients per (shape, schedule) from measured points: each
    {N,H,W,C,M,S,schedule,idx (array),ms}."""
    from scipy.optimize import least_squares
    out = {}
    groups: Dict[str, List[dict]] = {}
    for p in points:
        groups.setdefault(key_of(p["C"], p["M"], p["S"], p["schedule"]), []).append(p)
    for key, pts in groups.items():
        sch = pts[0]["schedule"]
        kind = "tiled" if sch == "tiled" else FUSED[(pts[0]["C"], pts[0]["M"], pts[0]["S"])]["kind"]
        feats = [features(np.asarray(p["idx"]), p["N"], p["H"], p["W"], p["C"], p["M"], p["S"], sch) for p in pts]
        y = np.array([p["ms"] * 1e3 for p in pts])
        names = ["F", "g1", "g2", "p"] if sch == "tiled" else ["t0", "c"] if kind == "stream" else ["t0", "w0", "a", "b", "c"]
        if sch != "tiled" and kind == "fused" and FUSED[(pts[0]["C"], pts[0]["M"], pts[0]["S"])]["PPW"] * pts[0]["S"] ** 2 > 64:
            names.append("d")
        x0 = np.full(len(names), 1.0)

        def resid(v):
            k = dict(zip(names, v))
            return np.array([_predict(f, k, sch, kind) for f in feats]) / y - 1.0

        r = least_squares(resid, x0, bounds=(0.0, np.inf))
        out[key] = {n: float(v) for n, v in zip(names, r.x)}
        out[key]["mape"] = float(np.mean(np.abs(resid(r.x))))
    return out


def _load_coeffs():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "latency_coeffs.json")
    if os.path.exists(path):
        COEFFS.update(json.load(open(path)))


_load_coeffs()


def points_from_bench(paths: Sequence[str]) -> List[dict]:
    """Measured sweep points out of bench.py JSON lines (index lists regenerated from their seeds)."""
    from . import synth
    pts = []
    for path in paths:
        d = json.load(open(path))
        sched_main = d["config"]["schedule"]
        for name, sweep in d["ratio_sweeps"].items():
            cfg = synth.CONFIGS[name]
            sch = sched_main if name in d["config"]["workload"] else ("stream" if (cfg.C, cfg.M, cfg.S) == (256, 64, 8) else "fused")
            sch = "fused" if sch == "stream" else sch
            for q in sweep:
                il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, q["r_mean"], seed=cfg.seed, structure=q["structure"])
                assert len(il) == q["active"]
                pts.append(dict(N=cfg.N, H=cfg.H, W=cfg.W, C=cfg.C, M=cfg.M, S=cfg.S, schedule=sch, idx=il,
                                ms=q["block_ms"], r_mean=q["r_mean"], structure=q["structure"], workload=name))
    return pts


if __name__ == "__main__":
    import sys
    pts = points_from_bench(sys.argv[1:])
    co = fit(pts)
    print(json.dumps(co, indent=1))
    for p in pts:
        pred = predict_us(p["idx"], p["N"], p["H"], p["W"], p["C"], p["M"], p["S"], p["schedule"], co)
        print("%-12s %-6s r=%.2f %-4s measured %7.1f us  predicted %7.1f us  %+5.1f%%" % (
            p["workload"], p["schedule"], p["r_mean"], p["structure"], p["ms"] * 1e3, pred, 100 * (pred / (p["ms"] * 1e3) - 1)))
