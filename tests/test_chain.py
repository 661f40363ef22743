"""The 29 sparse blocks of a ResNet-101 body as a chain: every block teacher-forced against the oracle.

A chain has no end-to-end parity (bf16 rounding differences would move later logits across the
threshold), so each block is checked on its own: the oracle is fed the block input the GPU actually
produced, the block's mask must match bit for bit (the margin guard says whether the comparison is
meaningful) and its output within the bf16 tolerance, with the ReLU after the add."""
import numpy as np
import pytest
import torch

from oracle import lasnet_oracle as O
from paper_2210_06223_amd import synth
from tests import _util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,sample", [(4, None), (128, (0, 77))], ids=["n4_every_image", "n128_two_sampled_images"])
def test_chain_blocks_teacher_forced(N, sample):
    from paper_2210_06223_amd import chain
    ch = chain.SparseChain(N)
    taken = []
    imgs = list(range(N)) if sample is None else list(sample)

    def tap(bi, x, mask, idx, count, out):
        sel = torch.tensor(imgs, device=x.device)
        taken.append((bi, x.index_select(0, sel).cpu(), mask.index_select(0, sel).cpu().numpy().copy(),
                      idx.cpu().numpy().copy(), int(count.item()), out.index_select(0, sel).cpu()))

    ch.run(tap=tap)
    torch.cuda.synchronize()
    assert len(taken) == 29
    for bi, x_t, mask_h, idx_h, cnt, out_t in taken:
        blk = ch.blocks[bi]
        S = blk["S"]
        print("chain block", bi, "stage", blk["stage"], "r", round(blk["r"], 3), "active", cnt, flush=True)
        q = lambda k: synth.bf16_bits_to_f32(synth.f32_to_bf16_bits(blk[k])).astype(np.float64)
        wts = (q("W1"), blk["b1"].astype(np.float64), q("W2"), blk["b2"].astype(np.float64), q("W3"),
               blk["b3"].astype(np.float64))
        x64 = x_t.to(torch.float64).numpy()
        assert (x64 >= 0).all()                                   # block inputs follow a ReLU
        # masker on the GPU's own input: logits in fp64 on both sides; margin guard as in the block tests
        logits = O.masker_logits(x64, blk["Wm"].astype(np.float64), ch.bm[bi], S)
        scale = float(np.abs(blk["Wm"]).sum() * x64.max())
        assert ch.margin[bi] > 1e-9 * scale, "block %d: masker margin too small for a meaningful mask comparison" % bi
        mask_o = (logits > 0.0).astype(np.uint8)
        assert np.array_equal(mask_h, mask_o), "block %d: mask differs" % bi
        P_img = mask_o[0].size
        ids_o = np.concatenate([np.flatnonzero(mask_o[i].reshape(-1)) + n * P_img for i, n in enumerate(imgs)])
        got_ids = idx_h[:cnt]
        keep = np.isin(got_ids // P_img, imgs)
        assert np.array_equal(got_ids[keep], ids_o.astype(np.int32)), "block %d: index list differs" % bi
        assert np.all(np.diff(got_ids) > 0) and cnt <= ch.N * P_img
        ref = O.sparse_bottleneck(x64, mask_o, S, *wts, post_relu=True)
        up = np.broadcast_to(O.upsample_mask(mask_o, S)[..., None], ref.shape)
        U.assert_block_close(out_t.cuda(), ref, x_t.cuda(), up, "bf16", "chain block %d" % bi)
