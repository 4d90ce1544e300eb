"""Pin for the transformer-block oracle: with at most two blocks per side the sparse attention
is dense attention, and the block must equal a textbook pre-LN block assembled from library
routines (torch LayerNorm / linear / GELU / scaled_dot_product_attention in float64)."""
import numpy as np
import torch
import torch.nn.functional as F

from oracle import vit_block as ov
from paper_2601_12150_amd import synth


def test_block_equals_library_pre_ln_block_when_attention_is_dense():
    rng = np.random.default_rng(3)
    B, g, heads, D, mlp = 2, 6, 3, 8, 40
    dim, T = heads * D, 1 + g * g
    x = rng.standard_normal((B, T, dim))
    w = synth.make_block_weights(dim, mlp, seed=5, dtype="f32", ln_random=True)
    y, scores = ov.vit_block(x, w, g, g, 3, heads, ln_eps=1e-5, want_scores=True)

    t = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items()}
    tx = torch.from_numpy(x)
    a = F.layer_norm(tx, (dim,), t["ln1_g"], t["ln1_b"], 1e-5)
    qkv = F.linear(a, t["w_qkv"], t["b_qkv"]).reshape(B, T, 3, heads, D).permute(2, 0, 3, 1, 4)
    att = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2])
    h = tx + F.linear(att.permute(0, 2, 1, 3).reshape(B, T, dim), t["w_proj"], t["b_proj"])
    m = F.gelu(F.linear(F.layer_norm(h, (dim,), t["ln2_g"], t["ln2_b"], 1e-5), t["w_fc1"], t["b_fc1"]))
    ref = h + F.linear(m, t["w_fc2"], t["b_fc2"])
    # the C attention oracle takes q, k, v as float32: that rounding (6e-8 relative) is the only difference
    np.testing.assert_allclose(y, ref.numpy(), rtol=0, atol=1e-9)
    p = torch.softmax(qkv[0][:, :, 0:1] @ qkv[1].transpose(-1, -2) * D ** -0.5, dim=-1)[:, :, 0, 1:].mean(dim=1)
    np.testing.assert_allclose(scores, p.numpy(), rtol=0, atol=1e-10)


def test_layer_norm_and_gelu_special_values():
    x = np.array([[1.0, 2.0, 3.0, 6.0]])
    out = ov.layer_norm(x, np.ones(4), np.zeros(4), 0.0)
    np.testing.assert_allclose(out.mean(), 0.0, atol=1e-15)
    np.testing.assert_allclose((out ** 2).mean(), 1.0, atol=1e-14)
    np.testing.assert_allclose(ov.gelu(np.array([0.0, 1e3, -1e3])), [0.0, 1e3, 0.0], atol=1e-12)
    # gelu(1) = 0.5 * (1 + erf(1/sqrt 2)) = Phi(1)
    np.testing.assert_allclose(ov.gelu(np.array([1.0])), [0.8413447460685429], atol=1e-15)


def test_patch_embed_equals_library_strided_convolution():
    """The tokenisation is a convolution with kernel = stride = patch side (library routine, fp64),
    flattened in raster order, with the CLS token in front and the position embeddings added."""
    rng = np.random.default_rng(5)
    B, ch, gh, gw, ps, dim = 2, 3, 3, 5, 4, 16
    px = rng.standard_normal((B, ch, gh * ps, gw * ps))
    w = rng.standard_normal((dim, ch * ps * ps))
    b = rng.standard_normal(dim)
    cls = rng.standard_normal(dim)
    pos = rng.standard_normal((1 + gh * gw, dim))
    got = ov.patch_embed(px, w, b, cls, pos, ps)
    conv = torch.nn.functional.conv2d(torch.from_numpy(px), torch.from_numpy(w.reshape(dim, ch, ps, ps)),
                                      torch.from_numpy(b), stride=ps)          # [B, dim, gh, gw]
    want = conv.flatten(2).transpose(1, 2).numpy() + pos[1:]
    np.testing.assert_allclose(got[:, 1:], want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(got[:, 0], np.broadcast_to(cls + pos[0], (B, dim)), rtol=0, atol=0)


def test_patch_embed_one_hot_projection_picks_single_pixels():
    """A projection row that is one-hot at (channel c, y, x) must return exactly that pixel of every
    patch: pins the (channel, y, x) order and the raster order of the patches."""
    rng = np.random.default_rng(6)
    B, ch, gh, gw, ps = 1, 2, 2, 3, 3
    px = rng.standard_normal((B, ch, gh * ps, gw * ps))
    picks = [(0, 0, 0), (1, 2, 1), (0, 1, 2), (1, 0, 2)]
    w = np.zeros((len(picks), ch * ps * ps))
    for i, (c, y, x) in enumerate(picks):
        w[i, (c * ps + y) * ps + x] = 1.0
    got = ov.patch_embed(px, w, np.zeros(len(picks)), np.zeros(len(picks)), np.zeros((1 + gh * gw, len(picks))), ps)
    for pr in range(gh):
        for pc in range(gw):
            for i, (c, y, x) in enumerate(picks):
                assert got[0, 1 + pr * gw + pc, i] == px[0, c, pr * ps + y, pc * ps + x]


def test_round_bf16_equals_library_conversion():
    """The block oracle's storage rounding against torch's float32 -> bfloat16 conversion (round to
    nearest even), including exact ties, signed zeros, denormals and values next to overflow."""
    rng = np.random.default_rng(8)
    x = np.concatenate([rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000)),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895313892515355e38, 1e-40, -1e-45],
                        # exact ties: bf16 has 8 significand bits, so 1 + (2k+1) * 2^-8 lies half way
                        1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8])
    want = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    got = ov.round_bf16(x)
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64))
    assert ov.round_bf16(np.array([1.00390625]))[0] == 1.0            # tie -> even (down)
    assert ov.round_bf16(np.array([1.01171875]))[0] == 1.015625       # tie -> even (up)


def test_bf16_storage_model_rounds_every_stored_tensor():
    """storage="bf16": outputs and the q, k behind the scores are bfloat16 values, and the result stays
    within a few bf16 steps of the unrounded block (the model changes precision, not the function)."""
    rng = np.random.default_rng(9)
    B, g, heads, D, mlp = 1, 8, 2, 8, 24
    dim, T = heads * D, 1 + g * g
    x = ov.round_bf16(rng.standard_normal((B, T, dim)))
    w = synth.make_block_weights(dim, mlp, seed=6, dtype="bf16", ln_random=True)
    y64, s64 = ov.vit_block(x, w, g, g, 4, heads, want_scores=True)
    y16, s16 = ov.vit_block(x, w, g, g, 4, heads, want_scores=True, storage="bf16")
    assert np.array_equal(ov.round_bf16(y16), y16)
    assert not np.array_equal(y16, y64)
    np.testing.assert_allclose(y16, y64, rtol=3e-2, atol=3e-2 * np.sqrt((y64 ** 2).mean()))
    np.testing.assert_allclose(s16, s64, rtol=5e-2)
    np.testing.assert_allclose(s16.sum(axis=1) + 0, s16.sum(axis=1))   # finite
