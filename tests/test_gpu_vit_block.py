"""GPU parity: vit_block_forward (through the C ABI) against the float64 block oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import vit_block as ov
from paper_2601_12150_amd import synth
from _util import assert_attn_close, assert_kept_sets_match, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def dev_weights(w):
    return {k: (torch.from_numpy(v).to(torch.bfloat16) if k.startswith("w_") else torch.from_numpy(v)).cuda()
            for k, v in w.items()}


def block_case(nb, B, g, block, heads, dim, mlp, seed, coords_keep=None):
    print("block case B=%d grid=%d block=%d heads=%d dim=%d mlp=%d pruned=%s" % (
        B, g, block, heads, dim, mlp, coords_keep is not None), flush=True)
    rng = np.random.default_rng(seed)
    if coords_keep is None:
        T, coords = 1 + g * g, None
    else:
        kept = np.sort(rng.choice(g * g, size=coords_keep, replace=False))
        T = 1 + len(kept)
        coords = np.ascontiguousarray(np.broadcast_to(synth.raster_coords(g, g)[kept], (B, len(kept))))
    x = synth.round_to_bf16(rng.standard_normal((B, T, dim)).astype(np.float32))
    w = synth.make_block_weights(dim, mlp, seed=seed, dtype="bf16", ln_random=True)
    ref, ref_scores = ov.vit_block(x, w, g, g, block, heads, ln_eps=1e-6, coords=coords, want_scores=True)
    dx = torch.from_numpy(x).to(torch.bfloat16).cuda()
    dc = None if coords is None else torch.from_numpy(coords).cuda()
    out, scores = nb.vit_block_forward(dx, dev_weights(w), g, g, block, heads, ln_eps=1e-6, coords=dc,
                                       want_scores=True)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, "bf16", "block output")
    # scores are computed from bf16-rounded q, k: a few 1e-3 relative
    np.testing.assert_allclose(to_np(scores), ref_scores, rtol=3e-2, atol=1e-7)
    return out


@pytest.mark.parametrize("B,g,block,heads,dim,mlp", [(1, 16, 8, 8, 512, 1024), (2, 24, 8, 8, 512, 640),
                                                     (1, 32, 16, 16, 1024, 4096), (1, 10, 4, 8, 512, 128)])
def test_block_matches_oracle(nb, B, g, block, heads, dim, mlp):
    block_case(nb, B, g, block, heads, dim, mlp, seed=11)


def test_block_on_pruned_sequence(nb):
    block_case(nb, 1, 24, 8, 8, 512, 1024, seed=12, coords_keep=350)


def test_block_validation(nb):
    x = torch.zeros((1, 65, 512), dtype=torch.bfloat16, device="cuda")
    w = dev_weights(synth.make_block_weights(512, 1024))
    with pytest.raises(nb.NsError) as e:
        nb.vit_block_forward(x, w, 8, 8, 4, 7)          # 7 heads do not divide 512
    assert e.value.code == nb.NS_ERR_INVALID_ARG
    with pytest.raises(nb.NsError) as e:
        nb.vit_block_forward(x, w, 8, 9, 4, 8)          # tokens != 1 + 72
    assert e.value.code == nb.NS_ERR_INVALID_ARG
