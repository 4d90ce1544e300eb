"""Several global tokens (paper, "Memory-Efficiency Optimization": a few designated global tokens
attend to, and are attended by, every token): G leading tokens, each a dense query row and a key
of every patch query; the importance score averages the G rows and the heads."""
import numpy as np
import pytest
import torch

import oracle
from oracle.vit_block import vit_block as oracle_block
from paper_2601_12150_amd import synth
from _util import assert_attn_close, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


@pytest.mark.parametrize("G,gh,gw,block,dtype,kernel", [
    (2, 16, 16, 8, "bf16", "attn_mfma_ragged_kernel"), (5, 20, 27, 8, "bf16", "attn_mfma_ragged_kernel"),
    (3, 32, 32, 16, "bf16", "attn_mfma_ragged_kernel"), (70, 12, 12, 4, "bf16", "attn_mfma_ragged_kernel"),
    (130, 9, 9, 8, "bf16", "attn_mfma_ragged_kernel"), (4, 14, 14, 7, "f32", "attn_generic_kernel"),
    (2, 10, 9, 4, "f32", "attn_generic_kernel")])
def test_attention_with_several_global_tokens(nb, G, gh, gw, block, dtype, kernel):
    B, H = 2, 3
    q, k, v = synth.small_case(400 + G, B, H, 64, gh, gw, dtype, n_global=G)
    ref = oracle.ns_attn(q, k, v, gh, gw, block, 0.125, n_global=G)
    dq, dk, dv = (to_dev(a, dtype) for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, block, n_global=G) == kernel
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, 0.125, want_cls=True, n_global=G)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, dtype, "G = %d" % G)        # global rows 0..G-1 included
    # by-products of every global row against the definition
    T = G + gh * gw
    s = 0.125 * np.einsum("bhgd,bhtd->bhgt", q[:, :, :G].astype(np.float64), k.astype(np.float64))
    np.testing.assert_allclose(to_np(logits).reshape(B, H, G, T), s, rtol=0, atol=2e-5)
    m = s.max(axis=-1, keepdims=True)
    ref_lse = (m + np.log(np.exp(s - m).sum(axis=-1, keepdims=True)))[..., 0]
    np.testing.assert_allclose(to_np(lse).reshape(B, H, G), ref_lse, rtol=0, atol=2e-5)
    # scores: mean over heads and global rows, both routes
    ref_scores = oracle.cls_scores(q, k, 0.125, n_global=G)
    s1 = nb.cls_scores(dq, dk, 0.125, n_global=G)
    s2 = nb.cls_scores_from_logits(logits, lse, n_global=G)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_np(s1), ref_scores, rtol=5e-5, atol=1e-10)
    np.testing.assert_allclose(to_np(s2), ref_scores, rtol=5e-5, atol=1e-10)
    assert torch.equal(s1, s2)


@pytest.mark.parametrize("force,G,gh,gw,block,gain", [
    ("sweep", 2, 24, 24, 8, 1.0), ("sweep", 8, 16, 40, 8, 1.0), ("sweep", 3, 20, 27, 8, 1.0), ("sweep", 5, 24, 16, 4, 1.0),
    ("sweep", 4, 19, 18, 2, 1.0), ("sweep", 3, 24, 24, 8, 14.0), ("sweep", 7, 8, 8, 8, 1.0),
    ("block", 2, 32, 32, 16, 1.0), ("block", 8, 48, 32, 16, 1.0), ("block", 3, 37, 21, 16, 1.0), ("block", 5, 70, 53, 32, 1.0),
    ("block", 4, 32, 48, 16, 14.0), ("block", 6, 5, 5, 64, 1.0)])
def test_tiled_kernels_with_several_global_tokens(nb, monkeypatch, force, G, gh, gw, block, gain):
    """Up to eight global tokens on the sweep and the block kernel (their K and V rows stay in LDS
    next to the first one's): grids the tiles divide and do not divide, windows 2-32, a block
    larger than the grid, and logits large enough (gain 14) to send query tiles through the
    running-maximum path.  The global rows come from the row kernel."""
    monkeypatch.setenv("NSATTN_KERNEL", force)
    B, H = 2, 3
    q, k, v = synth.small_case(500 + G, B, H, 64, gh, gw, "bf16", n_global=G)
    if gain != 1.0:
        q = synth.round_to_bf16(q * np.float32(gain))
    ref = oracle.ns_attn(q, k, v, gh, gw, block, 0.125, n_global=G)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    name = nb.ns_attn_patch_kernel_name(dq, gh, gw, block, n_global=G)
    assert name == ("attn_sweep_kernel" if force == "sweep" else "attn_block16_kernel")
    out, logits, lse, scores = nb.ns_attn_forward_scores(dq, dk, dv, gh, gw, block, 0.125, n_global=G)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, "bf16", "%s G = %d" % (force, G))
    ref_scores = oracle.cls_scores(q, k, 0.125, n_global=G)
    np.testing.assert_allclose(to_np(scores), ref_scores, rtol=5e-5, atol=1e-10)
    out2 = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, 0.125, n_global=G)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


def test_sweep_is_chosen_for_a_few_global_tokens_at_size(nb, monkeypatch):
    """A backbone with register tokens on a grid large enough to fill the chip: the tiled kernel is
    the default, nine or more global tokens go to the list kernel."""
    monkeypatch.delenv("NSATTN_KERNEL", raising=False)
    B, H, g, G = 2, 16, 64, 5
    q, k, v = synth.small_case(600, B, H, 64, g, g, "bf16", n_global=G)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, g, g, 8, n_global=G) == "attn_sweep_kernel"
    assert nb.ns_attn_patch_kernel_name(dq, g, g, 16, n_global=G) == "attn_block16_kernel"
    for block in (8, 16):
        ref = oracle.ns_attn(q, k, v, g, g, block, 0.125, n_global=G)
        out = nb.ns_attn_forward(dq, dk, dv, g, g, block, 0.125, n_global=G)
        torch.cuda.synchronize()
        assert_attn_close(to_np(out), ref, "bf16", "G = 5 on the 64 x 64 grid, block %d" % block)
    q9, k9, v9 = synth.small_case(601, 1, H, 64, g, g, "bf16", n_global=9)
    assert nb.ns_attn_patch_kernel_name(to_dev(q9, "bf16"), g, g, 8, n_global=9) == "attn_mfma_ragged_kernel"


def test_pruned_sequence_with_several_global_tokens(nb):
    G, g, block = 3, 30, 8
    rng = np.random.default_rng(9)
    kept = np.flatnonzero(rng.random(g * g) < 0.6)
    B, H = 2, 2
    q, k, v = synth.small_case(77, B, H, 64, 1, len(kept), "bf16", n_global=G)
    coords = np.ascontiguousarray(np.broadcast_to(synth.raster_coords(g, g)[kept], (B, len(kept))))
    ref = oracle.ns_attn(q, k, v, g, g, block, 0.125, coords=coords, n_global=G)
    out = nb.ns_attn_forward(*(to_dev(a, "bf16") for a in (q, k, v)), g, g, block, 0.125,
                             coords=torch.from_numpy(coords).cuda(), n_global=G)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, "bf16", "pruned, G = 3")


@pytest.mark.parametrize("G,dtype", [(2, "bf16"), (5, "f32")])
def test_filter_keeps_the_global_rows(nb, G, dtype):
    B, N, C, k = 3, 500, 128, 123
    rng = np.random.default_rng(G)
    scores = rng.random((B, N)).astype(np.float32)
    x = synth.round_to_bf16(rng.standard_normal((B, G + N, C)).astype(np.float32))
    kept, y, _ = nb.topk_filter(torch.from_numpy(scores).cuda(), k, x=to_dev(x, dtype), n_global=G)
    torch.cuda.synchronize()
    ref_kept = oracle.topk(scores, k)
    assert np.array_equal(kept.cpu().numpy(), ref_kept)
    ref_y = oracle.gather(x, ref_kept, n_global=G)
    assert np.array_equal(to_np(y), ref_y)


def test_block_and_stack_with_two_global_tokens(nb):
    G, g, block, H, dim, mlp = 2, 16, 8, 8, 512, 1024
    B, T = 2, G + g * g
    w = synth.make_block_weights(dim, mlp, seed=5, ln_random=True)
    rng = np.random.default_rng(12)
    x = synth.round_to_bf16(rng.standard_normal((B, T, dim)).astype(np.float32))
    ref, ref_scores = oracle_block(x, w, g, g, block, H, want_scores=True, n_global=G, storage="bf16")
    dw = {n: (torch.from_numpy(a).to(torch.bfloat16) if n.startswith("w_") else torch.from_numpy(a)).cuda()
          for n, a in w.items()}
    y, scores = nb.vit_block_forward(to_dev(x, "bf16"), dw, g, g, block, H, want_scores=True, n_global=G)
    torch.cuda.synchronize()
    got = to_np(y)
    assert_attn_close(got, ref, "bf16", "block with two global tokens")
    # (the block oracle in its bf16 storage model: what is left is the rare bf16 step where fp32 and
    # float64 accumulation round q or k differently)
    np.testing.assert_allclose(to_np(scores), ref_scores, rtol=5e-4, atol=0)
    # a stack of two such blocks with a pruning stage in between keeps both global rows
    keep = 100
    out, kept = nb.vit_forward(to_dev(x, "bf16"), [dw, dw], g, g, block, H, prune_after=1, keep_k=keep, n_global=G)
    torch.cuda.synchronize()
    assert out.shape == (B, G + keep, dim)
    kept_np = kept.cpu().numpy()
    assert np.array_equal(kept_np, oracle.topk(to_np(scores), keep))      # selection on the GPU's own scores
    x1 = oracle.gather(got, kept_np, n_global=G)                            # block 1 output, compacted
    coords = np.ascontiguousarray(synth.raster_coords(g, g)[kept_np])
    ref2 = oracle_block(x1, w, g, g, block, H, coords=coords, n_global=G, storage="bf16")
    assert_attn_close(to_np(out), ref2, "bf16", "second block on the pruned sequence")
