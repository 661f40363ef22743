"""The latency predictor (Sec. 3.3 / App. A re-parameterised for this library on MI355X): its replay of
the kernels' work split, and its predictions against the measured sweeps stored under profiles/."""
import os

import numpy as np

from paper_2210_06223_amd import latency_model as LM
from paper_2210_06223_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_replay_of_the_fused_kernels_work_split():
    cfg = synth.CONFIGS["stage3_b128"]
    idx = np.arange(0, cfg.P, 2, dtype=np.int32)                # 3136 of 6272 cells
    wgs = LM.simulate_fused(idx, cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S)
    assert len(wgs) == 256                                      # one round of one workgroup per CU
    assert sum(len(w) for w in wgs) >= 256
    out_blocks = sum(b2 for w in wgs for _, b2 in w)
    assert out_blocks * 16 >= len(idx) * cfg.S * cfg.S          # every active pixel is in some 16-row block
    # isolated cells (no shared window pixels): 16 of them need 16 * 16 rows > 160, so batches are cut
    iso = np.array([n * 49 + gy * 7 + gx for n in range(64) for gy in (0, 2, 4, 6) for gx in (0, 2, 4, 6)], np.int32)
    wgs = LM.simulate_fused(iso, cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S)
    assert all(b1 <= 10 for w in wgs for b1, _ in w)            # never more than R1MAX = 160 rows
    # an empty list costs nothing to replay
    assert LM.simulate_fused(np.zeros(0, np.int32), cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S) == []


def test_window_pixels_counts():
    assert len(LM.window_pixels([(0, 0, 0)], 2, 14, 14)) == 9          # corner patch: 3 x 3 in the image
    assert len(LM.window_pixels([(0, 3, 3)], 2, 14, 14)) == 16         # interior: 4 x 4
    assert len(LM.window_pixels([(0, 3, 3), (0, 3, 4)], 2, 14, 14)) == 24   # neighbours share 2 columns


def test_predictions_against_the_stored_sweeps():
    worst = 0.0
    n = 0
    for line in open(os.path.join(ROOT, "profiles", "ratio_sweeps_mi355x.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, sch, r, structure, active, measured, _ = line.split()
        cfg = synth.CONFIGS[name]
        il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, float(r), seed=cfg.seed, structure=structure)
        assert len(il) == int(active)
        pred = LM.predict_us(il, cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S, sch)
        worst = max(worst, abs(pred / float(measured) - 1.0))
        n += 1
    assert n >= 50 and worst < 0.15, worst


def test_predicted_latency_does_not_fall_when_more_is_active():
    cfg = synth.CONFIGS["stage4_b128"]
    prev = 0.0
    for r in (0.1, 0.3, 0.5, 0.8, 1.0):
        il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, r, seed=3, structure="blob")
        t = LM.predict_us(il, cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S, "tiled")
        assert t >= prev - 1e-9
        prev = t
