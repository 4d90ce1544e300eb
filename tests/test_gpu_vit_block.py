"""GPU parity: vit_block_forward (through the C ABI) against the float64 block oracle."""
import numpy as np
import pytest
import torch

import oracle
from oracle import vit_block as ov
from paper_2601_12150_amd import synth
from _util import assert_attn_close, assert_kept_sets_match, to_np

pytestmark = pytest.mark.gpu

# Importance scores of a whole block against the block oracle in its bf16 storage model: see block_case.
SCORE_RTOL = 5e-4


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def dev_weights(w):
    return {k: (torch.from_numpy(v).to(torch.bfloat16) if k.startswith("w_") else torch.from_numpy(v)).cuda()
            for k, v in w.items()}


def block_case(nb, B, g, block, heads, dim, mlp, seed, coords_keep=None, edit=None):
    print("block case B=%d grid=%d block=%d heads=%d dim=%d mlp=%d pruned=%s" % (
        B, g, block, heads, dim, mlp, coords_keep is not None), flush=True)
    rng = np.random.default_rng(seed)
    if coords_keep is None:
        T, coords = 1 + g * g, None
    else:
        kept = np.sort(rng.choice(g * g, size=coords_keep, replace=False))
        T = 1 + len(kept)
        coords = np.ascontiguousarray(np.broadcast_to(synth.raster_coords(g, g)[kept], (B, len(kept))))
    x = rng.standard_normal((B, T, dim)).astype(np.float32)
    if edit is not None:
        edit(x, rng)
    x = synth.round_to_bf16(x)
    w = synth.make_block_weights(dim, mlp, seed=seed, dtype="bf16", ln_random=True)
    # the oracle in its "bf16 storage" precision model: every tensor the block keeps in memory between
    # two steps is rounded to bf16 there as well, all arithmetic in float64
    ref, ref_scores = ov.vit_block(x, w, g, g, block, heads, ln_eps=1e-6, coords=coords, want_scores=True,
                                   storage="bf16")
    dx = torch.from_numpy(x).to(torch.bfloat16).cuda()
    dc = None if coords is None else torch.from_numpy(coords).cuda()
    out, scores = nb.vit_block_forward(dx, dev_weights(w), g, g, block, heads, ln_eps=1e-6, coords=dc,
                                       want_scores=True)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, "bf16", "block output")
    # q and k of both sides are bf16 values computed from the same bf16 inputs; they differ where
    # fp32 and float64 accumulation fall on different sides of a bf16 rounding boundary (about one
    # element in a thousand, by one bf16 step = 2^-8 of one of 64 products of a logit)
    rel = np.abs(to_np(scores) - ref_scores) / ref_scores
    print("scores: max relative deviation %.2e, mean %.2e" % (rel.max(), rel.mean()), flush=True)
    np.testing.assert_allclose(to_np(scores), ref_scores, rtol=SCORE_RTOL, atol=0)
    return out


@pytest.mark.parametrize("B,g,block,heads,dim,mlp", [(1, 16, 8, 8, 512, 1024), (2, 24, 8, 8, 512, 640),
                                                     (1, 32, 16, 16, 1024, 4096), (1, 10, 4, 8, 512, 128)])
def test_block_matches_oracle(nb, B, g, block, heads, dim, mlp):
    block_case(nb, B, g, block, heads, dim, mlp, seed=11)


def test_block_on_pruned_sequence(nb):
    block_case(nb, 1, 24, 8, 8, 512, 1024, seed=12, coords_keep=350)


def test_block_with_degenerate_rows(nb):
    """Rows that strain the normalisation: constant (variance 0), all zero, a mean of 100 standard deviations
    (a one-pass variance would cancel), single outlier channels, tiny amplitudes — the global token's row among them."""
    def edit(x, rng):
        x[:, 0] = 0.75                       # the global token: constant
        x[:, 5] = 0.0
        x[:, 9] += 100.0
        x[:, 17, 3] = 250.0
        x[:, 18, ::64] = -60.0
        x[:, 40:48] *= 1e-3
        x[:, 100:108] *= 30.0
    block_case(nb, 2, 16, 8, 8, 512, 1024, seed=13, edit=edit)


def test_block_validation(nb):
    x = torch.zeros((1, 65, 512), dtype=torch.bfloat16, device="cuda")
    w = dev_weights(synth.make_block_weights(512, 1024))
    with pytest.raises(nb.NsError) as e:
        nb.vit_block_forward(x, w, 8, 8, 4, 7)          # 7 heads do not divide 512
    assert e.value.code == nb.NS_ERR_INVALID_ARG
    with pytest.raises(nb.NsError) as e:
        nb.vit_block_forward(x, w, 8, 9, 4, 8)          # tokens != 1 + 72
    assert e.value.code == nb.NS_ERR_INVALID_ARG


@pytest.mark.parametrize("layers,after,keep_pct,g,block", [(4, 2, 60, 16, 8), (5, 4, 40, 16, 8), (3, 1, 20, 20, 8),
                                                           (3, 3, 50, 16, 8), (4, 2, 30, 32, 16)])
def test_stack_with_pruning_stage(nb, layers, after, keep_pct, g, block):
    """A stack with the pruning stage after block `after` (the paper's example: after the fourth
    layer) and keep ratios 20-60 % (discarded proportion p = 0.4-0.8).  The GPU's kept set must
    agree with the oracle's scores outside the tie band; the oracle then continues on the GPU's
    kept set, so the final outputs are comparable element by element."""
    B, heads, dim, mlp = 2, 8, 512, 640
    N, T = g * g, 1 + g * g
    keep = (N * keep_pct + 99) // 100
    rng = np.random.default_rng(21)
    x = synth.round_to_bf16(rng.standard_normal((B, T, dim)).astype(np.float32))
    ws = [synth.make_block_weights(dim, mlp, seed=30 + i, dtype="bf16", ln_random=True) for i in range(layers)]
    out, kept = nb.vit_forward(torch.from_numpy(x).to(torch.bfloat16).cuda(), [dev_weights(w) for w in ws],
                               g, g, block, heads, prune_after=after, keep_k=keep)
    torch.cuda.synchronize()
    kept_np = kept.cpu().numpy()

    h = x.astype(np.float64)
    for i in range(after):
        if i + 1 == after:
            h, scores = ov.vit_block(h, ws[i], g, g, block, heads, want_scores=True, storage="bf16")
        else:
            h = ov.vit_block(h, ws[i], g, g, block, heads, storage="bf16")
    ref_kept = oracle.topk(scores.astype(np.float32), keep)
    # kept sets agree outside the stated tie band (1e-3 relative around the k-th score)
    assert_kept_sets_match(kept_np, ref_kept, scores, keep)
    idx = np.concatenate([np.zeros((B, 1), dtype=np.int64), 1 + kept_np.astype(np.int64)], axis=1)
    h = np.take_along_axis(h, idx[:, :, None], axis=1)
    coords = np.stack([synth.raster_coords(g, g)[kept_np[b]] for b in range(B)])
    for i in range(after, layers):
        h = ov.vit_block(h, ws[i], g, g, block, heads, coords=coords, storage="bf16")
    assert_attn_close(to_np(out), h, "bf16", "stack output")


@pytest.mark.parametrize("layers,after,keep_pct,g,block", [(5, (1, 3), (70, 40), 16, 8), (6, (2, 3, 5), (80, 50, 20), 20, 8),
                                                           (4, (2, 4), (60, 60), 32, 16), (3, (1, 2), (50, 3), 16, 8)])
def test_stack_with_several_pruning_stages(nb, layers, after, keep_pct, g, block):
    """Several pruning stages (the paper's rule applied repeatedly): each stage ranks the patches still
    present by the scores of the block before it.  The oracle follows the GPU's kept set after every
    stage (obtained from the same stack cut off after that stage), checks it against its own scores
    outside the tie band, and the final outputs are compared element by element."""
    B, heads, dim, mlp = 2, 8, 512, 640
    N, T = g * g, 1 + g * g
    keeps = [(N * pc + 99) // 100 for pc in keep_pct]
    rng = np.random.default_rng(31)
    x = synth.round_to_bf16(rng.standard_normal((B, T, dim)).astype(np.float32))
    ws = [synth.make_block_weights(dim, mlp, seed=60 + i, dtype="bf16", ln_random=True) for i in range(layers)]
    dws = [dev_weights(w) for w in ws]
    dx = torch.from_numpy(x).to(torch.bfloat16).cuda()
    out, kept = nb.vit_forward_stages(dx, dws, g, g, block, heads, list(after), keeps)
    torch.cuda.synchronize()
    assert out.shape == (B, 1 + keeps[-1], dim)

    raster = synth.raster_coords(g, g)
    h = x.astype(np.float64)
    present = np.tile(np.arange(N, dtype=np.int64), (B, 1))          # original indices of the patches in the sequence
    coords = None
    stage = 0
    for i in range(layers):
        scoring = stage < len(after) and i + 1 == after[stage]
        if scoring:
            h, scores = ov.vit_block(h, ws[i], g, g, block, heads, coords=coords, want_scores=True, storage="bf16")
            # the GPU's survivors after this stage: the same stack cut off here
            _, kept_j = nb.vit_forward_stages(dx, dws[:i + 1], g, g, block, heads, list(after[:stage + 1]), keeps[:stage + 1])
            torch.cuda.synchronize()
            kept_orig = kept_j.cpu().numpy().astype(np.int64)
            assert np.all(np.diff(kept_orig, axis=1) > 0)
            # as positions in the current sequence
            local = np.stack([np.searchsorted(present[b], kept_orig[b]) for b in range(B)])
            assert all(np.array_equal(present[b][local[b]], kept_orig[b]) for b in range(B)), "survivors must come from the sequence"
            ref_local = oracle.topk(scores.astype(np.float32), keeps[stage])
            assert_kept_sets_match(local.astype(np.int32), ref_local, scores, keeps[stage])
            idx = np.concatenate([np.zeros((B, 1), dtype=np.int64), 1 + local], axis=1)
            h = np.take_along_axis(h, idx[:, :, None], axis=1)
            present = kept_orig
            coords = np.stack([raster[present[b]] for b in range(B)])
            stage += 1
        else:
            h = ov.vit_block(h, ws[i], g, g, block, heads, coords=coords, storage="bf16")
    assert np.array_equal(kept.cpu().numpy(), present)
    assert_attn_close(to_np(out), h, "bf16", "stack output after %d stages" % len(after))
    # one stage through this entry point is vit_forward
    out1, kept1 = nb.vit_forward_stages(dx, dws, g, g, block, heads, [after[0]], [keeps[0]])
    out2, kept2 = nb.vit_forward(dx, dws, g, g, block, heads, prune_after=after[0], keep_k=keeps[0])
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(kept1, kept2)


def test_stage_lists_are_validated(nb):
    x = torch.zeros((1, 65, 512), dtype=torch.bfloat16, device="cuda")
    ws = [dev_weights(synth.make_block_weights(512, 640, seed=i)) for i in range(3)]
    for after, keep in (([2, 2], [30, 20]), ([2, 1], [30, 20]), ([1, 2], [20, 30]), ([1], [65]), ([4], [10]), ([0], [10]), ([1], [0])):
        with pytest.raises(nb.NsError) as e:
            nb.vit_forward_stages(x, ws, 8, 8, 8, 8, after, keep)
        assert e.value.code == nb.NS_ERR_INVALID_ARG
    out, kept = nb.vit_forward_stages(x, ws, 8, 8, 8, 8, [], [])
    assert out.shape == x.shape and kept is None


def test_stack_pruning_of_a_long_sequence(nb):
    """More than 32768 patches: the stack's selection runs with several workgroups per image and
    takes its scratch from the stack's workspace.  The stack must keep exactly what topk_filter
    (checked against the oracle elsewhere) keeps from the same block's scores, and continue on it."""
    B, g, block, heads, dim, mlp = 1, 184, 8, 8, 512, 512
    N = g * g
    keep = (N * 60 + 99) // 100
    rng = np.random.default_rng(23)
    x = torch.from_numpy(synth.round_to_bf16(rng.standard_normal((B, 1 + N, dim)).astype(np.float32))).to(torch.bfloat16).cuda()
    ws = [dev_weights(synth.make_block_weights(dim, mlp, seed=50 + i)) for i in range(2)]
    out, kept = nb.vit_forward(x, ws, g, g, block, heads, prune_after=1, keep_k=keep)
    h, scores = nb.vit_block_forward(x, ws[0], g, g, block, heads, want_scores=True)
    coords = torch.from_numpy(synth.raster_coords(g, g).astype(np.int32)).cuda().repeat(B, 1).contiguous()
    kept2, y, cout = nb.topk_filter(scores, keep, x=h, coords=coords)
    torch.cuda.synchronize()
    assert np.array_equal(kept.cpu().numpy(), oracle.topk(scores.cpu().numpy(), keep))
    assert torch.equal(kept, kept2)
    out2 = nb.vit_block_forward(y, ws[1], g, g, block, heads, coords=cout)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)


@pytest.mark.parametrize("B,ch,gh,gw,ps,dim", [(2, 3, 20, 24, 14, 512), (1, 3, 16, 16, 16, 1024), (1, 1, 3, 5, 7, 128),
                                               (3, 3, 1, 1, 14, 256), (1, 3, 40, 33, 14, 1024)])
def test_patch_embedding_matches_oracle(nb, B, ch, gh, gw, ps, dim):
    """Tokenisation: 14-pixel patches (588 columns, padded to 640 inside) and 16-pixel patches (768),
    grids from one patch to more than a thousand, the CLS row, position embeddings as residual."""
    rng = np.random.default_rng(gh * 100 + gw)
    r = synth.round_to_bf16
    px = r(rng.standard_normal((B, ch, gh * ps, gw * ps)).astype(np.float32))
    w = r((rng.standard_normal((dim, ch * ps * ps)) * 0.05).astype(np.float32))
    b = (rng.standard_normal(dim) * 0.1).astype(np.float32)
    cls = r(rng.standard_normal(dim).astype(np.float32))
    pos = r((rng.standard_normal((1 + gh * gw, dim)) * 0.5).astype(np.float32))
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    out = nb.vit_embed(bf(px), bf(w), torch.from_numpy(b).cuda(), bf(cls), bf(pos), ps)
    torch.cuda.synchronize()
    ref = ov.patch_embed(px, w, b, cls, pos, ps)
    assert_attn_close(to_np(out), ref, "bf16", "patch embedding %dx%d, patch %d" % (gh, gw, ps))
    # and it feeds the stack: one block on the embedded tokens equals the block on the oracle's tokens
    if dim >= 512 and gh * gw >= 64:
        heads = dim // 64
        wb = synth.make_block_weights(dim, dim, seed=3)
        y = nb.vit_block_forward(out, dev_weights(wb), gh, gw, 8, heads)
        torch.cuda.synchronize()
        assert_attn_close(to_np(y), ov.vit_block(to_np(out).astype(np.float64), wb, gh, gw, 8, heads), "bf16",
                          "block on embedded tokens")


def test_stack_without_pruning_equals_repeated_blocks(nb):
    B, g, block, heads, dim, mlp = 1, 16, 8, 8, 512, 512
    rng = np.random.default_rng(22)
    x = torch.from_numpy(synth.round_to_bf16(rng.standard_normal((B, 1 + g * g, dim)).astype(np.float32))).to(torch.bfloat16).cuda()
    ws = [dev_weights(synth.make_block_weights(dim, mlp, seed=40 + i)) for i in range(3)]
    out, kept = nb.vit_forward(x, ws, g, g, block, heads)
    h = x
    for w in ws:
        h = nb.vit_block_forward(h, w, g, g, block, heads)
    torch.cuda.synchronize()
    assert kept is None and torch.equal(out, h)


def test_stack_feature_maps(nb):
    """Segmentation mode: sparse attention in every layer, no pruning, patch tokens after chosen
    blocks handed out in raster order.  Each map is compared with the oracle's chain of blocks
    (patch rows after blocks 1, 3 and 4, raster order) and, bit for bit, with the block-by-block run."""
    B, g, block, heads, dim, mlp = 2, 20, 8, 8, 512, 512       # 20 is not a multiple of 8
    rng = np.random.default_rng(23)
    x_np = synth.round_to_bf16(rng.standard_normal((B, 1 + g * g, dim)).astype(np.float32))
    x = torch.from_numpy(x_np).to(torch.bfloat16).cuda()
    ws_np = [synth.make_block_weights(dim, mlp, seed=50 + i) for i in range(4)]
    ws = [dev_weights(w) for w in ws_np]
    out, kept, taps = nb.vit_forward(x, ws, g, g, block, heads, tap_layers=[1, 3, 4])
    torch.cuda.synchronize()
    ref_h, ref_maps = x_np.astype(np.float64), {}
    for i, w in enumerate(ws_np):
        ref_h = ov.vit_block(ref_h, w, g, g, block, heads, storage="bf16")
        ref_maps[i + 1] = ref_h[:, 1:]
    for t, l in zip(taps, (1, 3, 4)):
        assert_attn_close(to_np(t), ref_maps[l], "bf16", "feature map after block %d" % l)
    assert_attn_close(to_np(out), ref_h, "bf16", "stack output")
    h, hs = x, []
    for w in ws:
        h = nb.vit_block_forward(h, w, g, g, block, heads)
        hs.append(h)
    torch.cuda.synchronize()
    assert kept is None and torch.equal(out, h)
    for t, l in zip(taps, (1, 3, 4)):
        assert t.shape == (B, g * g, dim) and torch.equal(t, hs[l - 1][:, 1:])
    # with a pruning stage, a map may be taken up to the pruning point and not after it
    keep = 150
    out2, kept2, taps2 = nb.vit_forward(x, ws, g, g, block, heads, prune_after=2, keep_k=keep, tap_layers=[2])
    torch.cuda.synchronize()
    assert torch.equal(taps2[0], hs[1][:, 1:]) and out2.shape == (B, 1 + keep, dim)
    with pytest.raises(nb.NsError) as e:
        nb.vit_forward(x, ws, g, g, block, heads, prune_after=2, keep_k=keep, tap_layers=[3])
    assert e.value.code == nb.NS_ERR_INVALID_ARG


@pytest.mark.parametrize("n", [256, 128])      # the 256 x 256 kernel and the 128 x 128 kernel
def test_gelu_epilogue_value_by_value(nb, n):
    """The GELU of the linear map's epilogue on chosen pre-activations: with the identity as weight and no bias
    the pre-activation is the input itself (exact in fp32), so every output is the bf16 rounding of gelu(x) — checked
    against the float64 erf form, relative to the value (the tail of negative x is where a form that subtracts loses
    its digits) plus the approximation's absolute error (1.5e-7 in erfc, times |x| / 2)."""
    M = 256
    vals = np.concatenate([np.linspace(-9.0, 9.0, M * n - 8), [0.0, -0.0, 1e-6, -1e-6, 40.0, -40.0, 1e4, -1e4]])
    x = synth.round_to_bf16(vals.astype(np.float32)).reshape(M, n)
    w = np.eye(n, dtype=np.float32)
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = nb.linear_forward(dev(x), dev(w), torch.zeros(n, device="cuda"), None, gelu=True)
    torch.cuda.synchronize()
    got = to_np(y).astype(np.float64)
    ref = ov.gelu(x.astype(np.float64))
    err = np.abs(got - ref)
    bound = 2.0 ** -8 * np.abs(ref) + 1e-7 * np.abs(x) + 1e-30
    worst = int(np.argmax(err / bound))
    assert np.all(err <= bound), (x.flat[worst], got.flat[worst], ref.flat[worst])
    assert np.all(got[x >= 0] >= 0) and np.all(got[x < 0] <= 0)


@pytest.mark.parametrize("M,N,K,gelu,res", [
    (1025, 1024, 1024, False, True),    # one extended row tile chain: 4 tiles, the last with a ninth slab
    (577, 512, 256, True, False),       # remainder 65: a partial tile of its own (3 slabs)
    (256, 256, 64, False, False),       # a single tile, a single k-slice
    (300, 768, 2048, True, True),       # remainder 44 -> partial tile with two slabs; long k
    (1154, 640, 512, False, True),      # N not a multiple of 256: the 128 x 128 kernel
    (37, 128, 64, True, True),          # fewer rows than any tile
    (9832, 4096, 128, False, True),     # more tiles than CUs: 19 rows of 256-row tiles, then 26 rows of 192-row tiles
    (7000, 4096, 64, False, False),     # 16 rows of each
    (12000, 2048, 64, False, True),     # 2 rows of 256-row tiles, then 60 of 192-row tiles
])
def test_linear_forward(nb, M, N, K, gelu, res):
    """The fused linear map against float64 matmul / erf GELU on the same bf16 inputs."""
    rng = np.random.default_rng(M + N + K)
    x = synth.round_to_bf16(rng.standard_normal((M, K)).astype(np.float32))
    w = synth.round_to_bf16((rng.standard_normal((N, K)) / np.sqrt(K)).astype(np.float32))
    b = rng.standard_normal(N).astype(np.float32)
    r = synth.round_to_bf16(rng.standard_normal((M, N)).astype(np.float32)) if res else None
    ref = x.astype(np.float64) @ w.astype(np.float64).T + b
    if gelu:
        ref = ov.gelu(ref)
    if res:
        ref = ref + r
    print("linear case M=%d N=%d K=%d gelu=%s residual=%s" % (M, N, K, gelu, res), flush=True)
    dev = lambda a: torch.from_numpy(a).to(torch.bfloat16).cuda()
    y = nb.linear_forward(dev(x), dev(w), torch.from_numpy(b).cuda(), None if r is None else dev(r), gelu=gelu)
    torch.cuda.synchronize()
    got = to_np(y).astype(np.float64)
    # one rounding to bf16 (2^-9 relative) on top of fp32 accumulation
    np.testing.assert_allclose(got, ref, rtol=2.0 ** -8, atol=1e-3)
