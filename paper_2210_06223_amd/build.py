"""Builds liblasnet.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2210_06223_amd.build`."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblasnet.so")
# The check build: the same sources with every hand-counted barrier of the matrix-core kernels waiting
# for all outstanding memory operations.  Only the tests load it (to compare the two bit for bit).
LIB_CHECK = os.path.join(PKG, "liblasnet_check.so")
CHECK_FLAGS = ("-DLASNET_DRAIN_AT_BARRIERS",)
SOURCES = ["tiled_stages.hip", "mfma_stage3.hip", "mfma_stage2.hip", "mfma_stage1.hip", "mfma_stage4.hip",   # slowest first
           "api.hip", "masker.hip", "bottleneck_generic.hip", "bottleneck_mfma.hip", "microbench.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 VALU ops
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


# The k-loops of the matrix-core kernels must be unrolled in full (their register rings are indexed
# by the loop counter; a ring that is not unrolled lands in scratch memory).  The long reductions of
# the tiled kernels exceed the compiler's default size limit for `#pragma unroll`.
PER_FILE_FLAGS = {"tiled_stages.hip": ["-mllvm", "-pragma-unroll-threshold=1048576"]}


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: liblasnet cannot be built")
    return exe


def _compile(cc, src, obj, extra_flags, verbose):
    cmd = [cc, *FLAGS, *PER_FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return obj


def _link(cc, objs, out, verbose):
    tmp = out + ".tmp"
    r = subprocess.run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs],
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    os.replace(tmp, out)
    if verbose:
        print("built", out)
    return out


def build_variants(variants, verbose: bool = True) -> None:
    """variants: (output path, build directory, extra flags) each; all files of all variants are
    compiled through one pool of workers, then each variant is linked."""
    cc = hipcc()
    jobs = []
    for out, bdir, extra in variants:
        os.makedirs(bdir, exist_ok=True)
        for src in SOURCES:
            jobs.append((src, os.path.join(bdir, os.path.splitext(src)[0] + ".o"), tuple(extra)))
    jobs.sort(key=lambda j: SOURCES.index(j[0]))          # slowest files first, over all variants
    with ThreadPoolExecutor(max_workers=min(8, len(jobs), os.cpu_count() or 1)) as ex:
        list(ex.map(lambda j: _compile(cc, j[0], j[1], j[2], verbose), jobs))
    for out, bdir, _ in variants:
        _link(cc, [os.path.join(bdir, os.path.splitext(src)[0] + ".o") for src in SOURCES], out, verbose)


def build_library(verbose: bool = True, extra_flags=(), out: str = LIB, build_dir: str = "") -> str:
    build_variants([(out, build_dir or os.path.join(PKG, "_build"), extra_flags)], verbose)
    return out


def build_all(verbose: bool = True) -> None:
    build_variants([(LIB, os.path.join(PKG, "_build"), ()),
                    (LIB_CHECK, os.path.join(PKG, "_build", "check"), CHECK_FLAGS)], verbose)


if __name__ == "__main__":
    build_all()
