"""The allocation-free entry point (lasnet_sparse_bottleneck_noalloc) against lasnet_sparse_bottleneck_ex.

Collected last on purpose (the name sorts after every other test file): the suite runs with -x."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2210_06223_amd import binding as B
from paper_2210_06223_amd import synth
from tests import _util as U


def test_shapes_beyond_the_scratch_array_are_refused_on_the_host():
    """Stage 4 needs 8.5 MiB of repacked weights: refused before any device call (fake pointers)."""
    L = B.lib()
    assert L.lasnet_packed_weights_bytes(B.LASNET_BF16, 2048, 512, 1) > B.LASNET_NOALLOC_MAX_PACKED_BYTES
    assert L.lasnet_packed_weights_bytes(B.LASNET_BF16, 1024, 256, 2) <= B.LASNET_NOALLOC_MAX_PACKED_BYTES
    p = ctypes.c_void_p(0x10000)
    x = B.lasnet_tensor(0x100000, 2, 7, 7, 2048, B.LASNET_BF16)
    o = B.lasnet_tensor(0x900000, 2, 7, 7, 2048, B.LASNET_BF16)
    st = L.lasnet_sparse_bottleneck_noalloc(ctypes.byref(x), p, p, 1, 512, p, p, p, p, p, p, ctypes.byref(o), 0, None)
    assert st == B.LASNET_ETOOBIG
    assert b"scratch" in L.lasnet_status_string(st)


@pytest.mark.gpu
def test_noalloc_entry_matches_the_allocating_one_twice_in_a_row():
    """Two calls in a row on the same GPU, the second with a smaller input and a smaller weight set, so
    it runs over what the first left in the shared scratch array; each against lasnet_sparse_bottleneck_ex
    bit for bit (same kernels, so nothing may differ), with the memory torch has reserved unchanged."""
    cases = [(synth.CONFIGS["stage3_b128"].with_(N=3, name="noalloc_s3"), B.LASNET_POST_RELU),        # 2.2 MiB of weights
             (synth.CONFIGS["stage2_b128"].with_(N=1, name="noalloc_s2"), B.LASNET_SKIP_IDENTITY),    # smaller map, 0.56 MiB
             (synth.CONFIGS["stage1_b64"].with_(N=1, S=4, name="noalloc_s1s4"), 0)]                   # 0.14 MiB
    prepared = []
    for cfg, flags in cases:
        inp = synth.make_block_inputs(cfg)
        d = U.dev_inputs(inp)
        il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.5, seed=cfg.seed + 7)
        idx = U.list_tensor(il, cfg.P)
        count = torch.tensor([len(il)], dtype=torch.int32, device="cuda")
        want = d["x"].clone()
        B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), out=want, flags=flags)
        got = d["x"].clone()
        prepared.append((cfg, flags, d, idx, count, want, got))
    torch.cuda.synchronize()
    for cfg, flags, d, idx, count, want, got in prepared:          # back to back, nothing in between
        print("noalloc", cfg.name, flush=True)
        B.lasnet_sparse_bottleneck_noalloc(d["x"], idx, count, cfg.S, *U.weights(d), out=got, flags=flags)
    torch.cuda.synchronize()
    for cfg, flags, d, idx, count, want, got in prepared:
        assert np.array_equal(U.bits(got), U.bits(want)), cfg.name
        assert not np.array_equal(U.bits(got), U.bits(d["x"])), cfg.name   # the block did run
