"""No-GPU checks of the boundary: the library loads, exports what include/lasnet.h declares,
and rejects bad arguments on the host before any HIP call."""
import ctypes
import os
import re

import pytest

from paper_2210_06223_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "lasnet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"LASNET_API\s+[\w\s\*]+?\b(lasnet_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(B.EXPORTS), names
    L = B.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert B.lasnet_version() >= 100
    assert L.lasnet_status_string(0) == b"ok"
    assert b"alias" in L.lasnet_status_string(B.LASNET_EALIAS)


def _t(n=1, h=8, w=8, c=16, dtype=B.LASNET_F32, data=0x1000):
    return B.lasnet_tensor(data, n, h, w, c, dtype)


def test_masker_argument_errors():
    L = B.lib()
    x = _t()
    p = ctypes.c_void_p(0x2000)
    call = lambda xx, wm, S, m=p, i=p, c=p: L.lasnet_masker(xx, wm, 0.0, S, 0.0, m, i, c, None)
    assert call(None, p, 2) == B.LASNET_EINVAL
    assert call(ctypes.byref(x), None, 2) == B.LASNET_EINVAL
    assert call(ctypes.byref(x), p, 0) == B.LASNET_EINVAL
    assert call(ctypes.byref(x), p, 3) == B.LASNET_ESHAPE          # 3 does not divide 8
    assert call(ctypes.byref(x), p, 2, m=None) == B.LASNET_EINVAL
    assert call(ctypes.byref(x), p, 2, c=None) == B.LASNET_EINVAL
    bad = _t(dtype=7)
    assert call(ctypes.byref(bad), p, 2) == B.LASNET_EINVAL
    assert L.lasnet_masker_logits(ctypes.byref(x), p, 0.0, 2, None, None) == B.LASNET_EINVAL
    # fused identity pass-through: the destination must match x and be another buffer
    ex = lambda po: L.lasnet_masker_ex(ctypes.byref(x), p, 0.0, 2, 0.0, p, p, p, ctypes.byref(po), None)
    assert ex(_t(data=0x1000)) == B.LASNET_EALIAS
    assert ex(_t(data=0x9000, c=32)) == B.LASNET_ESHAPE
    assert ex(_t(data=0x9000, dtype=B.LASNET_BF16)) == B.LASNET_ESHAPE
    assert ex(_t(data=0)) == B.LASNET_EINVAL


def test_block_argument_errors():
    L = B.lib()
    p = ctypes.c_void_p(0x2000)
    x, o = _t(), _t(data=0x9000)
    w = [p] * 6

    def call(xx, oo, S=2, M=4, idx=p, cnt=p, ws=w):
        return L.lasnet_sparse_bottleneck(ctypes.byref(xx), idx, cnt, S, M, *ws, ctypes.byref(oo), None)

    assert call(x, x) == B.LASNET_EALIAS
    assert call(x, _t(h=4, data=0x9000)) == B.LASNET_ESHAPE
    assert call(x, _t(dtype=B.LASNET_BF16, data=0x9000)) == B.LASNET_ESHAPE
    assert call(x, o, S=3) == B.LASNET_ESHAPE
    assert call(x, o, S=0) == B.LASNET_EINVAL
    assert call(x, o, M=0) == B.LASNET_EINVAL
    assert call(x, o, cnt=None) == B.LASNET_EINVAL                 # idx without count
    assert call(x, o, ws=[p, None, p, p, p, p]) == B.LASNET_EINVAL
    big = _t(h=16, w=16, c=4096)                                   # generic tile cannot hold M=8192 in LDS
    assert call(big, _t(h=16, w=16, c=4096, data=0x9000), S=16, M=8192) == B.LASNET_EUNSUPPORTED


def test_fast_path_query():
    import torch
    assert B.lasnet_has_fast_path(torch.bfloat16, 1024, 256, 2) == 1
    assert B.lasnet_has_fast_path(torch.bfloat16, 512, 128, 4) == 1
    assert B.lasnet_has_fast_path(torch.bfloat16, 256, 64, 8) == 1
    assert B.lasnet_has_fast_path(torch.float32, 1024, 256, 2) == 0
    assert B.lasnet_has_fast_path(torch.bfloat16, 64, 16, 4) == 0
    assert B.lasnet_has_fast_path(torch.float32, 64, 8192, 16) == B.LASNET_EUNSUPPORTED


def test_binding_rejects_host_tensors():
    import torch
    x = torch.zeros((1, 4, 4, 8))
    with pytest.raises(ValueError):
        B.lasnet_masker(x, torch.zeros(8), 0.0, 2)


def test_product_path_never_touches_the_oracle():
    """The oracle is test infrastructure: the package (binding, input generator, build script and
    every HIP source) must not import or include it; bench.py only in its cpu_baseline leg."""
    pkg = os.path.join(ROOT, "paper_2210_06223_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath or "__pycache__" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(import|from)\s+oracle|#include.*oracle|import_module\(.oracle", text, re.M), \
                    os.path.join(dirpath, f)
    bench = open(os.path.join(ROOT, "bench.py")).read()
    uses = [i for i, line in enumerate(bench.splitlines()) if re.search(r"\bimport\b.*\boracle\b|from oracle", line)]
    start = bench.splitlines().index("def cpu_baseline(cfg, inp, bm):")
    assert uses and all(i > start for i in uses)


def test_flag_and_status_values_match_the_header():
    text = open(os.path.join(ROOT, "include", "lasnet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    vals = {k: int(v) for k, v in re.findall(r"\b(LASNET_[A-Z0-9_]+)\s*=\s*(-?\d+)", text)}
    for name in ("LASNET_OK", "LASNET_EINVAL", "LASNET_ESHAPE", "LASNET_EUNSUPPORTED", "LASNET_EALIAS", "LASNET_EHIP",
                 "LASNET_ETOOBIG", "LASNET_F32", "LASNET_BF16", "LASNET_POST_RELU", "LASNET_FORCE_GENERIC",
                 "LASNET_SKIP_IDENTITY", "LASNET_FORCE_FUSED", "LASNET_FORCE_TILED"):
        assert name in vals, name
        assert getattr(B, name) == vals[name], name


def test_schedules_workspace_query_and_planned_entry_argument_errors():
    """Host-side answers about the two schedules: which shapes have a tiled one and what it needs, and
    what the explicit entry refuses before any device call (fake pointers throughout)."""
    L = B.lib()
    bf = B.LASNET_BF16
    # 14x14x1024 (one image per group) and 7x7x2048 (two per group): cell masks + y1 + y2
    n, hw, m = 128, 196, 256
    assert L.lasnet_workspace_bytes(bf, n, 14, 14, 1024, m, 2) == (6272 + 255) // 256 * 256 + 2 * n * hw * m * 2
    assert L.lasnet_workspace_bytes(bf, 5, 7, 7, 2048, 512, 1) == 256 + 5 * 49 * 512 * 2 + 3 * 2 * 49 * 512 * 2
    assert L.lasnet_workspace_bytes(bf, 4, 28, 28, 512, 128, 4) == 0          # fused only
    assert L.lasnet_workspace_bytes(bf, 4, 28, 28, 1024, 256, 2) == 0         # an image does not fit a group
    assert L.lasnet_workspace_bytes(B.LASNET_F32, 4, 14, 14, 1024, 256, 2) == 0
    p = ctypes.c_void_p(0x10000)
    x = B.lasnet_tensor(0x100000, 2, 14, 14, 1024, bf)
    o = B.lasnet_tensor(0x900000, 2, 14, 14, 1024, bf)

    def planned(packed=p, ws=ctypes.c_void_p(0x4000000), wsb=1 << 30, flags=B.LASNET_FORCE_TILED, xx=x, oo=o, S=2, M=256):
        return L.lasnet_sparse_bottleneck_planned(ctypes.byref(xx), p, p, None, S, M, packed, p, p, p, ctypes.byref(oo),
                                                  flags, ws, wsb, None)

    assert planned(packed=None) == B.LASNET_EINVAL
    assert planned(ws=None) == B.LASNET_EINVAL                                 # the tiled schedule needs a workspace
    assert planned(wsb=1024) == B.LASNET_EINVAL                                # too small
    assert planned(ws=ctypes.c_void_p(0x4000010)) == B.LASNET_EINVAL           # not 256-byte aligned
    x2 = B.lasnet_tensor(0x100000, 2, 28, 28, 512, bf)
    o2 = B.lasnet_tensor(0x900000, 2, 28, 28, 512, bf)
    assert planned(xx=x2, oo=o2, S=4, M=128) == B.LASNET_EUNSUPPORTED          # no tiled schedule to force
    # in place: refused where the one-kernel schedule would run
    assert planned(xx=x, oo=x, flags=B.LASNET_FORCE_FUSED) == B.LASNET_EALIAS
    assert planned(xx=x, oo=x, flags=0) == B.LASNET_EALIAS                     # 14x14x1024 defaults to the fused schedule
    half = B.lasnet_tensor(0x100000 + 4096, 2, 14, 14, 1024, bf)
    assert planned(xx=x, oo=half) == B.LASNET_EALIAS                           # overlapping, not the same
    st = L.lasnet_sparse_bottleneck_noalloc(ctypes.byref(x), p, p, 2, 256, p, p, p, p, p, p, ctypes.byref(o),
                                            B.LASNET_FORCE_TILED, None)
    assert st == B.LASNET_EUNSUPPORTED                                         # that entry never runs the tiled schedule


def test_microbenchmark_argument_errors():
    """Bad arguments are refused on the host (0 FLOPs / 0 bytes / LASNET_EINVAL) before any HIP call."""
    L = B.lib()
    vp = ctypes.c_void_p
    assert L.lasnet_microbench_mfma(0, vp(0x1000), None) == 0.0
    assert L.lasnet_microbench_mfma(10, None, None) == 0.0
    assert L.lasnet_microbench_weight_stream(None, 128 * 1024, 1, vp(0x1000), None) == 0.0
    assert L.lasnet_microbench_weight_stream(vp(0x1000), 100 * 1024, 1, vp(0x1000), None) == 0.0      # not whole 128 KiB
    assert L.lasnet_microbench_weight_stream(vp(0x1008), 128 * 1024, 1, vp(0x1000), None) == 0.0      # misaligned
    assert L.lasnet_microbench_weight_stream(vp(0x1000), 128 * 1024, 0, vp(0x1000), None) == 0.0
    assert L.lasnet_microbench_weight_stream(vp(0x1000), 2 << 30, 1, vp(0x1000), None) == 0.0          # beyond 1 GiB
    assert L.lasnet_microbench_copy(vp(0x1000), vp(0x2000), 24, None) == B.LASNET_EINVAL
    assert L.lasnet_microbench_copy(vp(0x1004), vp(0x2000), 32, None) == B.LASNET_EINVAL
