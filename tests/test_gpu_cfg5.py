"""GPU parity at the full size of the backbone workload: a 2048 x 2048 synthetic tile, 16-pixel
patches (128 x 128 grid + CLS = 16385 tokens), width 1024, 16 heads, MLP 4096, 8 x 8 blocks.
Tokenisation and the first two transformer blocks through the C ABI against the float64 oracle in its
bf16 storage model (paper, "Settings": ViT backbone; Methodology: sparse attention in every layer)."""
import time

import numpy as np
import pytest
import torch

import oracle
from oracle import vit_block as ov
from paper_2601_12150_amd import synth
from _util import assert_attn_close, assert_kept_sets_match, to_np

pytestmark = pytest.mark.gpu


def test_tile_embedding_and_first_two_blocks_at_full_size():
    from paper_2601_12150_amd import binding as nb
    side, ps, dim, mlp, heads, blk = 2048, 16, 1024, 4096, 16, 8
    g = side // ps
    N = g * g
    pixels, bg = synth.make_tile(seed=5, side=side, patch=ps, background=0.40)
    e = synth.make_embed_weights(dim, ps, N, seed=5)
    ws = [synth.make_block_weights(dim, mlp, seed=100 + i) for i in range(2)]
    print("tile: background %.3f; tokens %d" % (bg.mean(), 1 + N), flush=True)

    def dev(a, bf16=True):
        t = torch.from_numpy(a)
        return (t.to(torch.bfloat16) if bf16 else t).cuda()
    dws = [{k: dev(v, k.startswith("w_")) for k, v in w.items()} for w in ws]
    x = nb.vit_embed(dev(pixels), dev(e["w_patch"]), dev(e["b_patch"], False), dev(e["cls_token"]),
                     dev(e["pos_embed"]), ps)
    h1, s1 = nb.vit_block_forward(x, dws[0], g, g, blk, heads, want_scores=True)
    h2 = nb.vit_block_forward(h1, dws[1], g, g, blk, heads)
    stack, _ = nb.vit_forward(x, dws, g, g, blk, heads)
    torch.cuda.synchronize()
    assert torch.equal(stack, h2), "the stack runs the same two blocks"

    t0 = time.time()
    rx = ov.round_bf16(ov.patch_embed(pixels, e["w_patch"], e["b_patch"], e["cls_token"], e["pos_embed"], ps))
    print("oracle embedding %.1f s" % (time.time() - t0), flush=True)
    assert_attn_close(to_np(x), rx, "bf16", "tokens")
    t0 = time.time()
    r1, rs1 = ov.vit_block(rx, ws[0], g, g, blk, heads, want_scores=True, storage="bf16")
    print("oracle block 1 %.1f s" % (time.time() - t0), flush=True)
    assert_attn_close(to_np(h1), r1, "bf16", "block 1 output")
    # both sides computed q and k from their own tokenisation (bf16 values that differ by one
    # rounding step here and there), so the scores are compared to the tie band itself
    rel = np.abs(to_np(s1) - rs1) / rs1
    print("scores: max relative deviation %.2e, mean %.2e" % (rel.max(), rel.mean()), flush=True)
    assert rel.max() < 1e-3
    keep = (N * 60 + 99) // 100
    kept, _, _ = nb.topk_filter(s1, keep)
    assert_kept_sets_match(kept.cpu().numpy(), oracle.topk(rs1.astype(np.float32), keep), rs1, keep)
    t0 = time.time()
    r2 = ov.vit_block(r1, ws[1], g, g, blk, heads, storage="bf16")
    print("oracle block 2 %.1f s" % (time.time() - t0), flush=True)
    assert_attn_close(to_np(h2), r2, "bf16", "block 2 output")
