"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Integer outputs (mask, idx, count) and inactive positions must be bit-exact; block outputs
within 1e-4 relative (fp32) / 2e-2 relative (bf16 storage, fp32 accumulate).
"""
import numpy as np
import pytest
import torch

from oracle import lasnet_oracle as O
from paper_2210_06223_amd import binding as B
from paper_2210_06223_amd import synth
from tests import _util as U

pytestmark = pytest.mark.gpu


def _say(*a):
    print(*a, flush=True)


def _cfg(base, **kw):
    return synth.CONFIGS[base].with_(**kw)


def _tiled(cfg):
    """Whether the library runs this shape on the tiled schedule (three kernels and a workspace)."""
    return B.lib().lasnet_workspace_bytes(B.LASNET_BF16 if cfg.dtype == "bf16" else B.LASNET_F32,
                                          cfg.N, cfg.H, cfg.W, cfg.C, cfg.M, cfg.S) > 0


def _oracle_w(inp):
    d = inp.f64
    return (d["W1"], d["b1"], d["W2"], d["b2"], d["W3"], d["b3"])


# ------------------------------------------------------------------ masker
MASKER_CASES = [
    _cfg("tiny_f32"),
    _cfg("stage3_b1"),
    _cfg("stage3_b128", N=5, name="stage3_n5"),
    _cfg("stage1_b64", N=2, name="stage1_n2"),
    _cfg("stage2_b128", N=3, name="stage2_n3"),
    _cfg("stage4_b128", N=4, name="stage4_n4"),
    synth.BlockConfig("odd_c20_s3_f32", 2, 6, 9, 20, 12, 3, "f32", 0.5, 21),     # scalar-load path
    synth.BlockConfig("odd_c20_s1_bf16", 2, 5, 7, 20, 12, 1, "bf16", 0.3, 22),
    synth.BlockConfig("pixel_s1_manycells", 8, 32, 32, 8, 8, 1, "f32", 0.37, 23),  # P = 8192: 8 compaction rounds
    synth.BlockConfig("layer_skip_sH", 3, 8, 8, 16, 8, 8, "bf16", 0.34, 24),       # S = H: one cell per image
    # fp32 with 4 KiB patch rows: the row-split masker with 1, 2 and 4 waves per cell (S = 1: one row per cell), odd cell counts
    synth.BlockConfig("rows_f32_s1", 1, 5, 7, 1024, 16, 1, "f32", 0.45, 31),
    synth.BlockConfig("rows_f32_s2", 1, 6, 6, 512, 16, 2, "f32", 0.45, 28),
    synth.BlockConfig("rows_f32_s4", 1, 12, 12, 256, 16, 4, "f32", 0.45, 29),
    synth.BlockConfig("rows_f32_s8", 3, 8, 24, 128, 16, 8, "f32", 0.45, 30),
]


@pytest.mark.parametrize("cfg", MASKER_CASES, ids=lambda c: c.name)
def test_masker_matches_oracle_bit_exact(cfg):
    _say("masker", cfg)
    inp = synth.make_block_inputs(cfg)
    k = int(round(cfg.r * cfg.P))
    bm = U.calibrate(inp, k)
    d = U.dev_inputs(inp)
    mask_o, idx_o, count_o, logits_o = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
    assert count_o == k
    idx = torch.full((cfg.P,), -7, dtype=torch.int32, device="cuda")
    mask, idx, count = B.lasnet_masker(d["x"], d["Wm"], bm, cfg.S, 0.0, idx=idx)
    logits = B.lasnet_masker_logits(d["x"], d["Wm"], bm, cfg.S)
    torch.cuda.synchronize()
    assert int(count.item()) == count_o
    assert np.array_equal(mask.cpu().numpy(), mask_o)
    idx_h = idx.cpu().numpy()
    assert np.array_equal(idx_h[:count_o], idx_o)
    assert (idx_h[count_o:] == -7).all()                      # tail untouched
    assert np.allclose(logits.cpu().numpy(), logits_o, rtol=1e-12, atol=1e-13)


def test_masker_threshold_and_extremes():
    cfg = _cfg("stage2_b128", N=2)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    for k, thr in ((0, 0.0), (cfg.P, 0.0), (cfg.P // 3, 0.125), (7, -0.5)):
        bm = U.calibrate(inp, k, thr)
        mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, thr)
        assert count_o == k
        mask, idx, count = B.lasnet_masker(d["x"], d["Wm"], bm, cfg.S, thr)
        torch.cuda.synchronize()
        assert int(count.item()) == k
        assert np.array_equal(mask.cpu().numpy(), mask_o)
        assert np.array_equal(idx.cpu().numpy()[:k], idx_o)


def test_masker_unaligned_mask_buffer_and_many_rounds():
    """A mask buffer that is not 8-byte aligned takes the byte-wise compaction; P = 20000 cells
    needs three rounds of the 8-cells-per-thread one."""
    cfg = synth.BlockConfig("pixel_s1_20000", 5, 50, 80, 8, 8, 1, "bf16", 0.41, 25)
    inp = synth.make_block_inputs(cfg)
    k = int(round(cfg.r * cfg.P))
    bm = U.calibrate(inp, k)
    d = U.dev_inputs(inp)
    mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
    for off in (0, 1):
        buf = torch.zeros(cfg.P + 8, dtype=torch.uint8, device="cuda")
        mask = buf[off:off + cfg.P].view(cfg.N, cfg.G, cfg.GW)
        _, idx, count = B.lasnet_masker(d["x"], d["Wm"], bm, cfg.S, 0.0, mask=mask)
        torch.cuda.synchronize()
        assert int(count.item()) == count_o == k
        assert np.array_equal(mask.cpu().numpy(), mask_o)
        assert np.array_equal(idx.cpu().numpy()[:k], idx_o)


MASKER_EX_CASES = [
    _cfg("stage3_b128", N=3, name="s3_ex"),        # matrix-core block kernel, hoisted masker path
    _cfg("stage2_b128", N=2, name="s2_ex"),
    _cfg("stage1_b64", N=1, name="s1_ex"),
    _cfg("stage4_b128", N=3, name="s4_ex"),
    _cfg("tiny_f32"),                              # fp32, generic block kernel
    synth.BlockConfig("odd_c20_s3_f32_ex", 2, 6, 9, 20, 12, 3, "f32", 0.5, 26),     # scalar masker path
    synth.BlockConfig("odd_c24_s2_bf16_ex", 3, 4, 6, 24, 8, 2, "bf16", 0.4, 27),    # 16-byte pieces, ragged groups
    synth.BlockConfig("rows_f32_s4_ex", 1, 12, 12, 256, 16, 4, "f32", 0.45, 31),    # row-split masker, fp32, odd cell count
]


@pytest.mark.parametrize("cfg", MASKER_EX_CASES, ids=lambda c: c.name)
def test_masker_with_fused_identity_then_block_without_copy(cfg):
    """lasnet_masker_ex copies the inactive cells, lasnet_sparse_bottleneck_ex(SKIP_IDENTITY) writes the
    active ones: together every element of a poisoned out, against the oracle."""
    _say("masker_ex", cfg)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    for k in (int(round(cfg.r * cfg.P)), 0, cfg.P):
        bm = U.calibrate(inp, k)
        mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
        out = torch.full_like(d["x"], 768.0)                               # exact in bf16
        mask, idx, count = B.lasnet_masker_ex(d["x"], d["Wm"], bm, cfg.S, 0.0, pass_out=out)
        torch.cuda.synchronize()
        assert int(count.item()) == count_o == k
        assert np.array_equal(mask.cpu().numpy(), mask_o)
        assert np.array_equal(idx.cpu().numpy()[:k], idx_o)
        up = np.broadcast_to(O.upsample_mask(mask_o, cfg.S)[..., None].astype(bool), tuple(d["x"].shape))
        o = U.to_f64(out)
        assert np.array_equal(U.bits(out)[~up], U.bits(d["x"])[~up])      # inactive cells: x, bit for bit
        assert (o[up] == 768.0).all()                                      # active cells: not touched
        B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), out=out,
                                   flags=B.LASNET_SKIP_IDENTITY)
        torch.cuda.synchronize()
        ref = O.sparse_bottleneck(inp.f64["x"], mask_o, cfg.S, *_oracle_w(inp))
        U.assert_block_close(out, ref, d["x"], up, cfg.dtype, cfg.name)
    with pytest.raises(B.LasnetError) as e:
        B.lasnet_masker_ex(d["x"], d["Wm"], 0.0, cfg.S, 0.0, pass_out=d["x"])
    assert e.value.status == B.LASNET_EALIAS


def test_masker_empty_batch():
    x = torch.zeros((0, 8, 8, 16), dtype=torch.bfloat16, device="cuda")
    Wm = torch.zeros(16, device="cuda")
    count = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    _, _, count = B.lasnet_masker(x, Wm, 0.0, 2, count=count)
    torch.cuda.synchronize()
    assert int(count.item()) == 0


# ------------------------------------------------------------------ block
def _run_case(cfg, k=None, idx_np=None, flags=0, order="ascending", use_masker=True):
    """One parity case.  Either the masker picks k cells (bias from the oracle's logits) or
    idx_np is fed directly.  Returns nothing; asserts."""
    _say("block", cfg, "k", k, "flags", flags, "order", order, "masker", use_masker)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    w = U.weights(d)
    if use_masker:
        bm = U.calibrate(inp, k)
        mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
        mask, idx, count = B.lasnet_masker(d["x"], d["Wm"], bm, cfg.S, 0.0)
        assert np.array_equal(mask.cpu().numpy(), mask_o)
    else:
        mask_o = np.zeros(cfg.P, np.uint8)
        mask_o[idx_np] = 1
        mask_o = mask_o.reshape(cfg.N, cfg.G, cfg.GW)
        idx = torch.full((cfg.P,), 0, dtype=torch.int32, device="cuda")
        idx[: len(idx_np)] = torch.from_numpy(idx_np).cuda()
        count = torch.tensor([len(idx_np)], dtype=torch.int32, device="cuda")
    out = torch.full_like(d["x"], 777.0)                     # poison: every element must be written
    B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *w, out=out, flags=flags)
    torch.cuda.synchronize()
    ref = O.sparse_bottleneck(inp.f64["x"], mask_o, cfg.S, *_oracle_w(inp),
                              post_relu=bool(flags & B.LASNET_POST_RELU))
    up = np.broadcast_to(O.upsample_mask(mask_o, cfg.S)[..., None], ref.shape)
    U.assert_block_close(out, ref, d["x"], up, cfg.dtype, cfg.name)
    return out


def test_tiny_f32_config():
    _run_case(_cfg("tiny_f32"), k=8)


GENERIC_CASES = [
    synth.BlockConfig("gen_f32_c20_m12_s3", 2, 6, 9, 20, 12, 3, "f32", 0.5, 31),
    synth.BlockConfig("gen_bf16_c24_m8_s2", 3, 4, 6, 24, 8, 2, "bf16", 0.5, 32),
    synth.BlockConfig("gen_f32_s1_pixel", 1, 5, 5, 16, 8, 1, "f32", 0.4, 33),
    synth.BlockConfig("gen_bf16_sH_layerskip", 3, 4, 4, 32, 16, 4, "bf16", 0.34, 34),
]


@pytest.mark.parametrize("cfg", GENERIC_CASES, ids=lambda c: c.name)
def test_generic_kernel_odd_shapes(cfg):
    _run_case(cfg, k=int(round(cfg.r * cfg.P)))
    _run_case(cfg, k=int(round(cfg.r * cfg.P)), flags=B.LASNET_POST_RELU)


# every matrix-core instantiation, small N: several workgroup tiles and a ragged last tile
MFMA_CASES = [
    (_cfg("stage3_b128", N=3, name="s3_S2"), 71),             # 147 cells, 71 active: 8 full tiles + 7
    (_cfg("stage3_b128", N=3, S=7, name="s3_S7"), 5),         # 12 cells
    (_cfg("stage2_b128", N=2, name="s2_S4"), 49),             # 98 cells, PPW=4 -> ragged
    (_cfg("stage2_b128", N=2, S=7, name="s2_S7"), 17),        # 32 cells, PPW=2 -> ragged
    (_cfg("stage1_b64", N=1, name="s1_S8"), 20),              # 49 cells
    (_cfg("stage1_b64", N=1, S=4, name="s1_S4"), 118),        # 196 cells (Table 1 block: S=4, r=0.6), ragged
    (_cfg("stage1_b64", N=1, S=7, name="s1_S7"), 31),         # 64 cells, ragged
    (_cfg("stage4_b128", N=5, name="s4_S1"), 117),            # pixel-level patches: 245 cells, 8 tiles of <= 16
    # other granularities of the same stages (Sec. 3.2: S ranges over the divisors of H)
    (_cfg("stage3_b128", N=2, S=1, name="s3_S1"), 201),       # 392 pixel-level cells, tiles of <= 64
    (_cfg("stage2_b128", N=1, S=2, name="s2_S2"), 95),        # 196 cells
    (_cfg("stage2_b128", N=1, S=1, name="s2_S1"), 391),       # 784 cells, tiles of <= 24
    (_cfg("stage1_b64", N=1, S=2, name="s1_S2"), 401),        # 784 cells
    (_cfg("stage1_b64", N=1, S=1, name="s1_S1"), 1570),       # 3136 cells, tiles of <= 16
]


@pytest.mark.parametrize("cfg,k", MFMA_CASES, ids=lambda v: getattr(v, "name", str(v)))
def test_mfma_kernel_matches_oracle(cfg, k):
    assert B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, cfg.S) == 1
    _run_case(cfg, k=k)
    if _tiled(cfg):                                            # the shape has both schedules: each on request too
        _run_case(cfg, k=k, flags=B.LASNET_FORCE_FUSED)
        _run_case(cfg, k=k, flags=B.LASNET_FORCE_TILED)


@pytest.mark.parametrize("cfg,k", MFMA_CASES[:1] + MFMA_CASES[2:3] + MFMA_CASES[4:5] + MFMA_CASES[7:9] + MFMA_CASES[10:11],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_mfma_extremes_and_flags(cfg, k):
    _run_case(cfg, k=0)                                        # ratio 0: identity, bit-exact
    _run_case(cfg, k=cfg.P)                                    # ratio 1: every patch active
    _run_case(cfg, k=1)
    _run_case(cfg, k=k, flags=B.LASNET_POST_RELU)
    _run_case(cfg, k=k, flags=B.LASNET_FORCE_GENERIC)          # scalar kernel on the same shape
    if _tiled(cfg):
        for forced in (B.LASNET_FORCE_FUSED, B.LASNET_FORCE_TILED):
            for kk in (0, cfg.P, 1):
                _run_case(cfg, k=kk, flags=forced)
            _run_case(cfg, k=k, flags=forced | B.LASNET_POST_RELU)


@pytest.mark.parametrize("structure", ["iid", "blob"])
def test_index_order_does_not_matter_and_direct_lists(structure):
    cfg = _cfg("stage2_b128", N=4, name="s2_lists")
    asc = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.5, seed=5, structure=structure)
    shf = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.5, seed=5, structure=structure, order="shuffled")
    assert sorted(shf.tolist()) == asc.tolist() and shf.tolist() != asc.tolist()
    a = _run_case(cfg, idx_np=asc, use_masker=False)
    b = _run_case(cfg, idx_np=shf, use_masker=False, order="shuffled")
    assert np.array_equal(U.bits(a), U.bits(b))


def test_isolated_patches_overflow_the_shared_halo_buffer():
    """Cells two apart share no neighbour pixels: a 16-patch batch then needs more distinct
    rows than the kernel keeps, and it has to split the batch (and still be exact)."""
    cfg = _cfg("stage3_b128", N=3, name="s3_isolated")
    cells = [n * 49 + gy * 7 + gx for n in range(cfg.N) for gy in (0, 2, 4, 6) for gx in (0, 2, 4, 6)]
    _run_case(cfg, idx_np=np.array(cells, np.int32), use_masker=False)
    cfg = _cfg("stage2_b128", N=2, name="s2_isolated")
    cells = [n * 49 + gy * 7 + gx for n in range(cfg.N) for gy in (1, 3, 5) for gx in (0, 2, 4, 6)]
    _run_case(cfg, idx_np=np.array(cells, np.int32), use_masker=False)


def test_prepacked_weights_entry_point_matches_plain_one():
    cfg = _cfg("stage3_b128", N=3, name="s3_packed")
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.5, seed=11)
    idx = U.list_tensor(il, cfg.P)
    count = torch.tensor([len(il)], dtype=torch.int32, device="cuda")
    a = B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d))
    packed = B.lasnet_pack_weights(cfg.S, d["W1"], d["W2"], d["W3"])
    b = torch.full_like(d["x"], 3.0)
    B.lasnet_sparse_bottleneck_packed(d["x"], idx, count, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out=b)
    torch.cuda.synchronize()
    assert np.array_equal(U.bits(a), U.bits(b))
    mask = np.zeros(cfg.P, np.uint8); mask[il] = 1
    mask = mask.reshape(cfg.N, cfg.G, cfg.GW)
    ref = O.sparse_bottleneck(inp.f64["x"], mask, cfg.S, *_oracle_w(inp))
    up = np.broadcast_to(O.upsample_mask(mask, cfg.S)[..., None], ref.shape)
    U.assert_block_close(b, ref, d["x"], up, cfg.dtype, cfg.name)
    # shapes without a matrix-core kernel are refused, not silently served by another path
    assert B.lib().lasnet_packed_weights_bytes(B.LASNET_BF16, 64, 16, 4) == 0
    assert B.lib().lasnet_packed_weights_bytes(B.LASNET_F32, 1024, 256, 2) == 0


def test_all_active_null_index_list_equals_dense_oracle():
    cfg = _cfg("stage3_b128", N=2, name="s3_null_idx")
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    out = torch.full_like(d["x"], 777.0)
    B.lasnet_sparse_bottleneck(d["x"], None, None, cfg.S, *U.weights(d), out=out)
    torch.cuda.synchronize()
    ref = O.dense_bottleneck(inp.f64["x"], *_oracle_w(inp))
    U.assert_block_close(out, ref, d["x"], np.ones(ref.shape, bool), cfg.dtype, cfg.name)


def test_full_batches_of_the_largest_size():
    """More cells than 256 workgroups x 24: runs of 29-31 patches, i.e. batches of 8 output row blocks
    (conv3 over two row groups), which batch 128 never reaches.  Every cell active, as a list and as NULL."""
    cfg = _cfg("stage3_b128", N=160, name="s3_n160_all_active")
    out_list = _run_case(cfg, idx_np=np.arange(cfg.P, dtype=np.int32), use_masker=False)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    out_null = torch.full_like(d["x"], 777.0)
    B.lasnet_sparse_bottleneck(d["x"], None, None, cfg.S, *U.weights(d), out=out_null)
    torch.cuda.synchronize()
    assert np.array_equal(U.bits(out_list), U.bits(out_null))
    # and a ratio at which runs of ~23 patches mix 5- and 6-block batches with cut ones
    il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.75, seed=77)
    _run_case(cfg, idx_np=il, use_masker=False)


DENSE_CASES = [
    _cfg("tiny_f32"),
    _cfg("stage3_b128", N=2, name="dense_s3"),
    _cfg("stage2_b128", N=1, name="dense_s2"),
    _cfg("stage1_b64", N=1, name="dense_s1"),
    _cfg("stage4_b128", N=2, name="dense_s4"),
    synth.BlockConfig("dense_gen_bf16", 2, 6, 4, 24, 8, 2, "bf16", 1.0, 41),
]


@pytest.mark.parametrize("cfg", DENSE_CASES, ids=lambda c: c.name)
def test_dense_block_matches_oracle(cfg):
    _say("dense", cfg)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    for flags in (0, B.LASNET_POST_RELU):
        out = torch.full_like(d["x"], 777.0)
        B.lasnet_dense_bottleneck(d["x"], *U.weights(d), out=out, flags=flags)
        torch.cuda.synchronize()
        ref = O.dense_bottleneck(inp.f64["x"], *_oracle_w(inp), post_relu=bool(flags))
        U.assert_block_close(out, ref, d["x"], np.ones(ref.shape, bool), cfg.dtype, cfg.name)


def test_skip_identity_flag_leaves_inactive_untouched():
    cfg = _cfg("stage1_b64", N=1, name="s1_skipid")
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    idx_np = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.4, seed=9)
    idx = U.list_tensor(idx_np, cfg.P)
    count = torch.tensor([len(idx_np)], dtype=torch.int32, device="cuda")
    out = torch.full_like(d["x"], 5.0)
    B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), out=out,
                               flags=B.LASNET_SKIP_IDENTITY)
    torch.cuda.synchronize()
    mask = np.zeros(cfg.P, np.uint8); mask[idx_np] = 1
    up = O.upsample_mask(mask.reshape(cfg.N, cfg.G, cfg.GW), cfg.S).astype(bool)
    o = U.to_f64(out)
    assert (o[~up] == 5.0).all() and not (o[up] == 5.0).all()


def test_errors_on_device_tensors():
    cfg = _cfg("tiny_f32")
    d = U.dev_inputs(synth.make_block_inputs(cfg))
    idx = torch.zeros(cfg.P, dtype=torch.int32, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(B.LasnetError) as e:
        B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), out=d["x"])
    assert e.value.status == B.LASNET_EALIAS
    with pytest.raises(B.LasnetError) as e:
        B.lasnet_sparse_bottleneck(d["x"], idx, count, 3, *U.weights(d))
    assert e.value.status == B.LASNET_ESHAPE
    # the list's storage must have room for every cell (the kernels request it together with the count)
    with pytest.raises(ValueError):
        B.lasnet_sparse_bottleneck(d["x"], idx[: cfg.P - 1].contiguous(), count, cfg.S, *U.weights(d))


# ------------------------------------------------------------------ full size, as bench.py launches it
def test_headline_workload_full_size_matches_oracle():
    """ResNet-101 stage 3, 14x14x1024, M=256, S=2, N=128, r=0.5: masker -> index list -> block,
    device-resident count, every output element against the oracle."""
    cfg = synth.CONFIGS["stage3_b128"]
    assert _tiled(cfg)
    _run_case(cfg, k=cfg.P // 2)
    _run_case(cfg, k=cfg.P // 2, flags=B.LASNET_FORCE_TILED)


@pytest.mark.parametrize("name", ["stage3_b128", "stage2_b128", "stage1_b64", "stage4_b128"])
def test_full_size_workloads_as_the_benchmark_launches_them(name):
    """The step bench.py times, at full size: lasnet_masker_ex (identity pass-through into out) then
    the block with LASNET_SKIP_IDENTITY through the prepacked-weights entry; every element of a
    poisoned out against the oracle, masks and index list bit-exact."""
    cfg = synth.CONFIGS[name]
    _say("full size", cfg)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    k = int(round(cfg.r * cfg.P))
    bm = U.calibrate(inp, k)
    mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
    out = torch.full_like(d["x"], 768.0)
    mask, idx, count = B.lasnet_masker_ex(d["x"], d["Wm"], bm, cfg.S, 0.0, pass_out=out)
    packed = B.lasnet_pack_weights(cfg.S, d["W1"], d["W2"], d["W3"])
    B.lasnet_sparse_bottleneck_packed(d["x"], idx, count, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"],
                                      out=out, flags=B.LASNET_SKIP_IDENTITY)
    torch.cuda.synchronize()
    assert int(count.item()) == count_o == k
    assert np.array_equal(mask.cpu().numpy(), mask_o)
    assert np.array_equal(idx.cpu().numpy()[:k], idx_o)
    ref = O.sparse_bottleneck(inp.f64["x"], mask_o, cfg.S, *_oracle_w(inp))
    up = np.broadcast_to(O.upsample_mask(mask_o, cfg.S)[..., None], ref.shape)
    U.assert_block_close(out, ref, d["x"], up, cfg.dtype, cfg.name)


# ------------------------------------------------------------------ batch 1, non-square maps, list hygiene
def test_block_at_batch_one():
    """One stage-3 image (49 cells): most workgroups get a single patch."""
    cfg = synth.CONFIGS["stage3_b1"]
    _run_case(cfg, k=24)
    _run_case(cfg, k=25, flags=B.LASNET_POST_RELU)


NONSQUARE_CASES = [
    (synth.BlockConfig("s3_S2_6x10", 3, 6, 10, 1024, 256, 2, "bf16", 0.5, 51), 23),     # 45 cells
    (synth.BlockConfig("s2_S4_8x12", 2, 8, 12, 512, 128, 4, "bf16", 0.5, 52), 7),       # 12 cells
    (synth.BlockConfig("s4_S1_3x5", 5, 3, 5, 2048, 512, 1, "bf16", 0.5, 53), 37),       # 75 cells
    (synth.BlockConfig("s1_S8_8x24", 2, 8, 24, 256, 64, 8, "bf16", 0.5, 54), 3),        # streaming kernel, 6 cells
]


@pytest.mark.parametrize("cfg,k", NONSQUARE_CASES, ids=lambda v: getattr(v, "name", str(v)))
def test_mfma_kernels_on_non_square_maps(cfg, k):
    assert B.lasnet_has_fast_path(torch.bfloat16, cfg.C, cfg.M, cfg.S) == 1
    _run_case(cfg, k=k)
    _run_case(cfg, k=cfg.P)
    if _tiled(cfg):
        for forced in (B.LASNET_FORCE_FUSED, B.LASNET_FORCE_TILED):
            _run_case(cfg, k=k, flags=forced)
            _run_case(cfg, k=cfg.P, flags=forced)


@pytest.mark.parametrize("cfg", [_cfg("stage3_b128", N=2, name="s3_hyg"), _cfg("stage1_b64", N=1, name="s1_hyg"),
                                 _cfg("tiny_f32")], ids=lambda c: c.name)
def test_count_beyond_capacity_and_invalid_entries(cfg):
    """count[0] > P is read as P; entries that are not cells of the map are ignored (the kernels
    check them, so a bad list cannot send a load or store outside the buffers)."""
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    w = U.weights(d)
    f, _, _ = O.residual_branch(inp.f64["x"], *_oracle_w(inp))
    # (1) a full list with an overstated count == every cell active
    idx = torch.arange(cfg.P, dtype=torch.int32, device="cuda")
    count = torch.tensor([cfg.P + 5], dtype=torch.int32, device="cuda")
    out = torch.full_like(d["x"], 777.0)
    B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *w, out=out)
    torch.cuda.synchronize()
    ones = np.ones((cfg.N, cfg.G, cfg.GW), np.uint8)
    ref = O.masked_output(inp.f64["x"], f, ones, cfg.S)
    U.assert_block_close(out, ref, d["x"], np.ones(ref.shape, bool), cfg.dtype, cfg.name)
    # (2) valid entries mixed with invalid ones, and a run of invalid ones long enough to fill a batch
    good = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.4, seed=77)
    room = cfg.P - len(good)                                   # the list's capacity is P entries
    bad = np.array([-1, cfg.P, cfg.P + 123, -2**31, 2**31 - 1] * 8, np.int32)[: max(0, room - 5)]
    mixed = np.concatenate([bad[:3], good[: len(good) // 2], bad, good[len(good) // 2:], bad[:2]]).astype(np.int32)
    assert len(good) < len(mixed) <= cfg.P
    mask = np.zeros(cfg.P, np.uint8); mask[good] = 1
    mask = mask.reshape(cfg.N, cfg.G, cfg.GW)
    idx = U.list_tensor(mixed, cfg.P)
    count = torch.tensor([len(mixed)], dtype=torch.int32, device="cuda")
    out = torch.full_like(d["x"], 777.0)
    B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *w, out=out)
    torch.cuda.synchronize()
    ref = O.masked_output(inp.f64["x"], f, mask, cfg.S)
    up = np.broadcast_to(O.upsample_mask(mask, cfg.S)[..., None], ref.shape)
    U.assert_block_close(out, ref, d["x"], up, cfg.dtype, cfg.name)


# ------------------------------------------------------------------ ratio sweep at full size
@pytest.mark.parametrize("name", ["stage2_b128", "stage3_b128", "stage4_b128"])
def test_ratio_sweep_index_lists_at_full_size(name):
    """The latency-against-ratio sweep as bench.py launches it (index lists with Beta-distributed
    per-image ratios, iid cells and one blob per image, fed straight to the prepacked entry with the
    identity pass-through skipped): every list against the oracle.  F(x) does not depend on the mask,
    so the oracle computes it once."""
    cfg = synth.CONFIGS[name]
    _say("ratio sweep", cfg)
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    f, _, _ = O.residual_branch(inp.f64["x"], *_oracle_w(inp))
    packed = B.lasnet_pack_weights(cfg.S, d["W1"], d["W2"], d["W3"])
    for r in (0.1, 0.25, 0.5, 0.75, 1.0):
        for structure in ("iid", "blob"):
            il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, r, seed=cfg.seed, structure=structure)
            _say("  r", r, structure, len(il))
            mask = np.zeros(cfg.P, np.uint8); mask[il] = 1
            mask = mask.reshape(cfg.N, cfg.G, cfg.GW)
            idx = torch.zeros((cfg.P,), dtype=torch.int32, device="cuda")
            idx[: len(il)] = torch.from_numpy(il).cuda()
            count = torch.tensor([len(il)], dtype=torch.int32, device="cuda")
            ref = O.masked_output(inp.f64["x"], f, mask, cfg.S)
            up = np.broadcast_to(O.upsample_mask(mask, cfg.S)[..., None], ref.shape)
            for flags in ((B.LASNET_FORCE_FUSED, B.LASNET_FORCE_TILED) if _tiled(cfg) else (0,)):
                out = d["x"].clone()                               # what the masker's pass-through leaves
                B.lasnet_sparse_bottleneck_packed(d["x"], idx, count, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"],
                                                  out=out, flags=B.LASNET_SKIP_IDENTITY | flags)
                torch.cuda.synchronize()
                U.assert_block_close(out, ref, d["x"], up, cfg.dtype, "%s r=%g %s flags %d" % (cfg.name, r, structure, flags))


# ------------------------------------------------------------------ the check build
def test_check_build_with_drained_barriers_is_bit_identical(monkeypatch):
    """The matrix-core kernels keep global->LDS loads in flight across barriers and wait for them with
    counts worked out by hand from the program order of each wave's memory operations.  The check build
    of the same sources waits for everything at those barriers.  If a count were off (say after a
    compiler moved a load), the production build would read stale LDS and differ from it."""
    from paper_2210_06223_amd import build as _build
    alt = B.load_library(_build.LIB_CHECK)
    assert alt is not B.lib()
    for cfg, k in MFMA_CASES + NONSQUARE_CASES:
        _say("check build", cfg.name)
        inp = synth.make_block_inputs(cfg)
        d = U.dev_inputs(inp)
        il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, k / cfg.P, seed=cfg.seed + 1000)
        idx = U.list_tensor(il, cfg.P)
        count = torch.tensor([len(il)], dtype=torch.int32, device="cuda")
        for flags in ((B.LASNET_FORCE_FUSED, B.LASNET_FORCE_TILED) if _tiled(cfg) else (0,)):
            outs = []
            for L in (B.lib(), alt):
                monkeypatch.setattr(B, "_lib", L)
                outs.append(B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), flags=flags))
                torch.cuda.synchronize()
            monkeypatch.undo()
            assert np.array_equal(U.bits(outs[0]), U.bits(outs[1])), (cfg.name, flags)


# ------------------------------------------------------------------ the explicit entry (caller's workspace and mask)
@pytest.mark.parametrize("cfg", [_cfg("stage3_b128", N=5, name="s3_planned"), _cfg("stage4_b128", N=7, name="s4_planned"),
                                 _cfg("stage3_b128", N=3, S=7, name="s3S7_planned"),
                                 _cfg("stage2_b128", N=2, name="s2_planned")], ids=lambda c: c.name)
def test_planned_entry_with_callers_workspace_and_mask(cfg):
    """lasnet_sparse_bottleneck_planned: packed weights, workspace and (optionally) the masker's byte mask
    from the caller.  With and without the mask, and shuffled lists, the output is the same bits; and it
    matches the oracle."""
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    k = int(round(cfg.r * cfg.P))
    bm = U.calibrate(inp, k)
    mask_o, idx_o, count_o, _ = O.masker(inp.f64["x"], inp.f64["Wm"], bm, cfg.S, 0.0)
    mask, idx, count = B.lasnet_masker(d["x"], d["Wm"], bm, cfg.S, 0.0)
    packed = B.lasnet_pack_weights(cfg.S, d["W1"], d["W2"], d["W3"])
    need = B.lasnet_workspace_bytes(d["x"], cfg.M, cfg.S)
    assert (need > 0) == _tiled(cfg)
    ws = torch.empty(need + 256, dtype=torch.uint8, device="cuda") if need else None
    forced = B.LASNET_FORCE_TILED if need else 0               # the three-kernel schedule wherever the shape has one
    if ws is not None:
        ws = ws[(-ws.data_ptr()) % 256:][:need]
    outs = []
    for m in (None, mask):
        out = torch.full_like(d["x"], 777.0)
        out.copy_(d["x"])
        B.lasnet_sparse_bottleneck_planned(d["x"], idx, count, m, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out, ws,
                                           flags=B.LASNET_SKIP_IDENTITY | forced)
        torch.cuda.synchronize()
        outs.append(out)
    perm = torch.randperm(k, device="cuda")
    idx_s = idx.clone(); idx_s[:k] = idx[:k][perm]
    out = d["x"].clone()
    B.lasnet_sparse_bottleneck_planned(d["x"], idx_s, count, None, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"], out, ws,
                                       flags=B.LASNET_SKIP_IDENTITY | forced)
    torch.cuda.synchronize()
    outs.append(out)
    assert np.array_equal(U.bits(outs[0]), U.bits(outs[1])) and np.array_equal(U.bits(outs[0]), U.bits(outs[2]))
    ref = O.sparse_bottleneck(inp.f64["x"], mask_o, cfg.S, *_oracle_w(inp))
    up = np.broadcast_to(O.upsample_mask(mask_o, cfg.S)[..., None], ref.shape)
    U.assert_block_close(outs[0], ref, d["x"], up, cfg.dtype, cfg.name)
    if need:                                                   # a workspace that is too small is refused
        with pytest.raises(B.LasnetError) as e:
            B.lasnet_sparse_bottleneck_planned(d["x"], idx, count, None, cfg.S, cfg.M, packed, d["b1"], d["b2"], d["b3"],
                                               out, ws[: need - 256], flags=forced)
        assert e.value.status == B.LASNET_EINVAL


# ------------------------------------------------------------------ in place (tiled schedule only)
@pytest.mark.parametrize("cfg,flags", [(_cfg("stage4_b128", N=5, name="s4_inplace"), 0),
                                       (_cfg("stage3_b128", N=4, name="s3_inplace"), B.LASNET_FORCE_TILED)],
                         ids=lambda v: getattr(v, "name", str(v)))
def test_in_place_update_on_the_tiled_schedule(cfg, flags):
    """out == x: the tiled schedule updates the active patches in place (its last kernel touches only
    their own elements, after the kernel that reads neighbours); same bits as out of place, and the
    oracle's result.  The fused schedule refuses."""
    inp = synth.make_block_inputs(cfg)
    d = U.dev_inputs(inp)
    il = synth.make_index_list(cfg.N, cfg.G, cfg.GW, 0.5, seed=cfg.seed + 3)
    idx = U.list_tensor(il, cfg.P)
    count = torch.tensor([len(il)], dtype=torch.int32, device="cuda")
    for post in (0, B.LASNET_POST_RELU):
        want = B.lasnet_sparse_bottleneck(d["x"], idx, count, cfg.S, *U.weights(d), flags=flags | post)
        xin = d["x"].clone()
        B.lasnet_sparse_bottleneck(xin, idx, count, cfg.S, *U.weights(d), out=xin, flags=flags | post)
        torch.cuda.synchronize()
        assert np.array_equal(U.bits(xin), U.bits(want))
    mask = np.zeros(cfg.P, np.uint8); mask[il] = 1
    mask = mask.reshape(cfg.N, cfg.G, cfg.GW)
    ref = O.sparse_bottleneck(inp.f64["x"], mask, cfg.S, *_oracle_w(inp), post_relu=True)
    up = np.broadcast_to(O.upsample_mask(mask, cfg.S)[..., None], ref.shape)
    U.assert_block_close(xin, ref, d["x"], up, cfg.dtype, cfg.name)
    # dense block in place
    xin = d["x"].clone()
    B.lasnet_dense_bottleneck(xin, *U.weights(d), out=xin, flags=flags)
    want = B.lasnet_dense_bottleneck(d["x"], *U.weights(d), flags=flags)
    torch.cuda.synchronize()
    assert np.array_equal(U.bits(xin), U.bits(want))
    # the one-kernel schedule cannot; overlapping but different buffers never
    with pytest.raises(B.LasnetError) as e:
        B.lasnet_sparse_bottleneck(xin, idx, count, cfg.S, *U.weights(d), out=xin, flags=B.LASNET_FORCE_FUSED)
    assert e.value.status == B.LASNET_EALIAS
    big = torch.zeros(d["x"].numel() + 8 * cfg.C, dtype=torch.bfloat16, device="cuda")
    a = big[: d["x"].numel()].view_as(d["x"]); b = big[8 * cfg.C:].view_as(d["x"])
    with pytest.raises(B.LasnetError) as e:
        B.lasnet_sparse_bottleneck(a, idx, count, cfg.S, *U.weights(d), out=b, flags=flags)
    assert e.value.status == B.LASNET_EALIAS
