"""Host-side pieces of bench.py: the one-GPU refusal and the counter-profile bookkeeping (no GPU needed)."""
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_source_signature_follows_the_kernel_sources(tmp_path, monkeypatch):
    sig = bench.source_signature()
    assert re.fullmatch(r"[0-9a-f]{16}", sig)
    assert sig == bench.source_signature()
    # a copy of the tree's csrc with one byte more gives another signature
    pkg = tmp_path / "paper_2210_06223_amd" / "csrc"
    pkg.mkdir(parents=True)
    src = os.path.join(ROOT, "paper_2210_06223_amd", "csrc")
    for f in os.listdir(src):
        (pkg / f).write_bytes(open(os.path.join(src, f), "rb").read())
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    assert bench.source_signature() == sig
    with open(pkg / "common.hpp", "ab") as fh:
        fh.write(b"\n")
    assert bench.source_signature() != sig


def test_stored_traffic_is_used_only_for_the_sources_it_was_measured_on(tmp_path, monkeypatch):
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    (tmp_path / "paper_2210_06223_amd" / "csrc").mkdir(parents=True)
    (tmp_path / "paper_2210_06223_amd" / "csrc" / "k.hip").write_text("kernel")
    (tmp_path / "profiles").mkdir()
    sig = bench.source_signature()
    f = tmp_path / "profiles" / "bench_w_hbm_traffic_pmc.txt"
    assert bench.stored_traffic("w", "fused") == (None, None)          # no file
    f.write_text("# notes\nTRAFFIC_BYTES_PER_LAUNCH fused 123456 sources %s\n" % sig)
    assert bench.stored_traffic("w", "fused") == (123456, os.path.join("profiles", "bench_w_hbm_traffic_pmc.txt"))
    assert bench.stored_traffic("w", "tiled") == (None, None)          # another schedule's line only
    (tmp_path / "paper_2210_06223_amd" / "csrc" / "k.hip").write_text("kernel, edited")
    val, src = bench.stored_traffic("w", "fused")
    assert val is None and "stale" in src


def test_committed_traffic_profiles_carry_a_machine_readable_line():
    for w in ("stage3_b128", "stage4_b128", "stage2_b128", "stage1_b64"):
        txt = open(os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic_pmc.txt" % w)).read()
        assert re.search(r"^TRAFFIC_BYTES_PER_LAUNCH (fused|tiled|stream) \d+ sources [0-9a-f]{16}$", txt, re.M), w
        assert "rocprofv3 --pmc FETCH_SIZE" in txt and "rocprofv3 --pmc WRITE_SIZE" in txt
