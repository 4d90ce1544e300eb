"""GPU parity: ns_attn_forward (through the C ABI) against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_12150_amd import synth
from _util import assert_attn_close, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def run_case(nb, seed, B, H, gh, gw, block, dtype, scale=0.125, strided=False):
    print("case seed=%d B=%d H=%d grid=%dx%d block=%d %s strided=%s" % (seed, B, H, gh, gw, block, dtype, strided),
          flush=True)
    q, k, v = synth.small_case(seed, B, H, 64, gh, gw, dtype)
    ref = oracle.ns_attn(q, k, v, gh, gw, block, scale)
    if strided:
        # q, k, v as views of one fused [B,T,3,H,D] projection, out as [B,T,H,D]
        T = q.shape[2]
        fused = torch.empty((B, T, 3, H, 64), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                            device="cuda")
        for i, a in enumerate((q, k, v)):
            fused[:, :, i] = to_dev(a, dtype).permute(0, 2, 1, 3)
        dq, dk, dv = (fused[:, :, i].permute(0, 2, 1, 3) for i in range(3))
        out_store = torch.empty((B, T, H, 64), dtype=fused.dtype, device="cuda")
        out = out_store.permute(0, 2, 1, 3)
        nb.ns_attn_forward(dq, dk, dv, gh, gw, block, scale, out=out)
    else:
        dq, dk, dv = (to_dev(a, dtype) for a in (q, k, v))
        out = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, scale)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, dtype, "attention")
    return out


# shape-generic kernel: odd block sizes, ragged last blocks, single-block grids, fp32 and bf16
@pytest.mark.parametrize("gh,gw,block,dtype", [
    (14, 14, 7, "f32"), (10, 9, 4, "f32"), (5, 5, 8, "f32"), (12, 20, 4, "bf16"), (9, 9, 3, "bf16"),
    (17, 13, 5, "bf16"), (24, 24, 12, "f32"), (16, 16, 8, "f32"), (3, 70, 2, "bf16")])
def test_generic_kernel(nb, monkeypatch, gh, gw, block, dtype):
    monkeypatch.setenv("NSATTN_KERNEL", "generic")     # bf16 would otherwise go to the list kernel
    run_case(nb, 101, 2, 3, gh, gw, block, dtype)


# MFMA kernel over per-block token lists on complete grids: block sides that do not divide the grid
# (short last blocks), block sides other than 8 and 16 (several runs of 64 per block for the large
# ones, nearly empty tiles for the small ones), a block that covers the whole grid
@pytest.mark.parametrize("gh,gw,block", [
    (20, 27, 8), (37, 21, 16), (12, 20, 4), (9, 9, 3), (17, 13, 5), (3, 70, 2), (30, 30, 2), (25, 25, 7),
    (40, 40, 64), (70, 72, 64), (33, 50, 32), (26, 26, 12), (5, 5, 8), (1, 1, 8), (1, 130, 16)])
def test_list_kernel_on_complete_grids(nb, gh, gw, block):
    q, k, v = synth.small_case(303, 2, 2, 64, gh, gw, "bf16")
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, block) == "attn_mfma_ragged_kernel"
    run_case(nb, 303, 2, 2, gh, gw, block, "bf16")


def test_list_kernel_strided_views(nb):
    run_case(nb, 304, 2, 4, 27, 22, 8, "bf16", scale=0.3, strided=True)


# MFMA kernel: 8x8 blocks (one tile each) and 16x16 blocks (four tiles each)
@pytest.mark.parametrize("gh,gw,block", [(16, 16, 8), (24, 40, 8), (8, 8, 8), (8, 24, 8), (32, 32, 16),
                                         (16, 48, 16), (48, 48, 8)])
def test_mfma_kernel(nb, gh, gw, block):
    run_case(nb, 202, 2, 3, gh, gw, block, "bf16")


def test_mfma_kernel_strided_views_and_other_scale(nb):
    run_case(nb, 203, 2, 4, 24, 24, 8, "bf16", scale=0.3, strided=True)


def test_generic_kernel_strided_views(nb):
    run_case(nb, 204, 1, 2, 10, 9, 4, "f32", strided=True)


def test_large_logits_do_not_overflow(nb):
    q, k, v = synth.small_case(7, 1, 2, 64, 16, 16, "bf16")
    q = synth.round_to_bf16(q * 12.0)
    ref = oracle.ns_attn(q, k, v, 16, 16, 8, 1.0)
    out = nb.ns_attn_forward(*(to_dev(a, "bf16") for a in (q, k, v)), 16, 16, 8, 1.0)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    assert_attn_close(to_np(out), ref, "bf16", "large logits")


@pytest.mark.parametrize("dtype,block", [("bf16", 8), ("f32", 4), ("bf16", 16)])
def test_pruned_sequence(nb, dtype, block):
    g = 32
    rng = np.random.default_rng(5)
    N = g * g
    keep = rng.random(N) < 0.55
    r, c = np.divmod(np.arange(N), g)
    keep[(r // block == 1) & (c // block == 1)] = False          # one block completely empty
    lone = (r // block == 0) & (c // block == g // block - 1)
    keep[lone] = False
    keep[np.flatnonzero(lone)[0]] = True                          # one block with a single token
    kept = np.flatnonzero(keep)
    B, H = 2, 2
    q, k, v = synth.small_case(31, B, H, 64, 1, len(kept), dtype)
    coords = np.ascontiguousarray(np.broadcast_to(synth.raster_coords(g, g)[kept], (B, len(kept))))
    ref = oracle.ns_attn(q, k, v, g, g, block, 0.125, coords=coords)
    dcoords = torch.from_numpy(coords).cuda()
    out = nb.ns_attn_forward(*(to_dev(a, dtype) for a in (q, k, v)), g, g, block, 0.125, coords=dcoords)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out), ref, dtype, "pruned sequence")


@pytest.mark.parametrize("g,block,shuffle,gain", [(30, 8, False, 1.0), (30, 5, True, 1.0), (20, 3, False, 1.0),
                                                  (32, 8, True, 12.0), (48, 16, True, 1.0), (40, 12, False, 1.0),
                                                  (50, 32, True, 6.0)])
def test_pruned_sequence_mfma_kernel(nb, monkeypatch, g, block, shuffle, gain):
    """bf16, head_dim 64: the MFMA kernel for pruned sequences.  Covers grids the block does not
    divide, blocks of more than 64 tokens (several runs per block, the last one partly filled),
    survivors in arbitrary sequence order, logits large enough to need the running maximum, and
    agreement with the fp32 FMA kernel on the same inputs."""
    rng = np.random.default_rng(g * 100 + block)
    N = g * g
    keep = rng.random(N) < 0.6
    r, c = np.divmod(np.arange(N), g)
    keep[(r // block == 0) & (c // block == 0)] = False            # an empty corner block
    kept = np.flatnonzero(keep)
    if shuffle:
        kept = rng.permutation(kept)
    B, H = 2, 3
    q, k, v = synth.small_case(77 + block, B, H, 64, 1, len(kept), "bf16")
    q = synth.round_to_bf16(q * gain)
    coords = np.ascontiguousarray(np.broadcast_to(synth.raster_coords(g, g)[kept], (B, len(kept))))
    ref = oracle.ns_attn(q, k, v, g, g, block, 0.125, coords=coords)
    dcoords = torch.from_numpy(coords).cuda()
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    out = nb.ns_attn_forward(dq, dk, dv, g, g, block, 0.125, coords=dcoords)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    assert_attn_close(to_np(out), ref, "bf16", "pruned sequence, MFMA kernel")
    monkeypatch.setenv("NSATTN_KERNEL", "generic")
    out_g = nb.ns_attn_forward(dq, dk, dv, g, g, block, 0.125, coords=dcoords)
    torch.cuda.synchronize()
    assert_attn_close(to_np(out_g), ref, "bf16", "pruned sequence, FMA kernel")


@pytest.mark.parametrize("variant,gh,gw", [(None, 24, 24), ("sweep", 24, 24), ("sweep", 16, 40), ("sweep", 8, 8),
                                           ("sweep", 40, 8), ("persist", 24, 24), ("mfma", 24, 24)])
def test_cls_by_products_and_determinism(nb, monkeypatch, variant, gh, gw):
    """Global-query by-products (raw logits, log-sum-exp) and its output row, for every way they are
    produced: the chunked row kernel, and the sweep kernel that computes them on the way."""
    if variant:
        monkeypatch.setenv("NSATTN_KERNEL", variant)
    q, k, v = synth.small_case(55, 2, 4, 64, gh, gw, "bf16")
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    out1, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, 8, 0.125, want_cls=True)
    out2 = nb.ns_attn_forward(dq, dk, dv, gh, gw, 8, 0.125)
    out3 = nb.ns_attn_forward(dq, dk, dv, gh, gw, 8, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(out1, out2) and torch.equal(out2, out3), "results must be bit-identical across runs"
    ref = oracle.ns_attn(q, k, v, gh, gw, 8, 0.125)
    assert_attn_close(to_np(out1)[:, :, :1], ref[:, :, :1], "bf16", "global query row")
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, 0.125, want_logits=True)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=2e-5)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=2e-5)


@pytest.mark.parametrize("gh,gw,gain", [(20, 27, 1.0), (9, 9, 1.0), (8, 100, 1.0), (17, 8, 1.0), (1, 1, 1.0), (5, 5, 1.0),
                                        (43, 60, 1.0), (12, 30, 14.0), (63, 65, 1.0)])
def test_sweep_on_grids_8_does_not_divide(nb, monkeypatch, gh, gw, gain):
    """The sweep kernel with short blocks at the right and bottom edge: patch rows, the global
    query's row and its by-products; gain 14 makes weights overflow the fixed exponent reference,
    so edge blocks also go through the running-maximum path."""
    monkeypatch.setenv("NSATTN_KERNEL", "sweep")
    q, k, v = synth.small_case(66, 2, 3, 64, gh, gw, "bf16")
    q = synth.round_to_bf16(q * gain)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, 8) == "attn_sweep_kernel"
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, 8, 0.125, want_cls=True)
    out2 = nb.ns_attn_forward(dq, dk, dv, gh, gw, 8, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    assert np.isfinite(to_np(out)).all()
    ref = oracle.ns_attn(q, k, v, gh, gw, 8, 0.125)
    assert_attn_close(to_np(out), ref, "bf16", "sweep on %dx%d" % (gh, gw))
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, 0.125, want_logits=True)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=2e-5 * gain)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=2e-5 * gain)


@pytest.mark.parametrize("gh,gw,gain", [(20, 27, 1.0), (37, 21, 1.0), (16, 50, 1.0), (33, 16, 1.0), (1, 1, 1.0), (5, 70, 1.0),
                                        (45, 60, 1.0), (19, 30, 14.0), (3, 3, 1.0)])
def test_block_kernel_on_grids_16_does_not_divide(nb, monkeypatch, gh, gw, gain):
    """The kernel for 16x16 blocks with short blocks at the right and bottom edge (query tiles
    with few or no rows of their own, key tiles partly or wholly made of copies); gain 14 sends
    edge tiles through the running-maximum path as well."""
    monkeypatch.setenv("NSATTN_KERNEL", "block")
    q, k, v = synth.small_case(67, 2, 3, 64, gh, gw, "bf16")
    q = synth.round_to_bf16(q * gain)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, 16) == "attn_block16_kernel"
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, 16, 0.125, want_cls=True)
    out2 = nb.ns_attn_forward(dq, dk, dv, gh, gw, 16, 0.125)
    torch.cuda.synchronize()
    assert torch.equal(out, out2)
    assert np.isfinite(to_np(out)).all()
    ref = oracle.ns_attn(q, k, v, gh, gw, 16, 0.125)
    assert_attn_close(to_np(out), ref, "bf16", "block kernel on %dx%d" % (gh, gw))
    # the global query's row is computed on the way: its by-products
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, 0.125, want_logits=True)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=2e-5 * gain)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=2e-5 * gain)


@pytest.mark.parametrize("gh,gw,block,gain", [(64, 64, 32, 1.0), (96, 128, 32, 1.0), (70, 53, 32, 1.0), (37, 21, 32, 1.0),
                                              (128, 64, 64, 1.0), (100, 75, 64, 1.0), (150, 40, 48, 1.0), (5, 5, 64, 1.0),
                                              (50, 70, 32, 14.0), (16, 16, 32, 1.0)])
def test_block_kernel_with_blocks_of_several_squares(nb, monkeypatch, gh, gw, block, gain):
    """Block sides 32, 48 and 64 on the block kernel: a 16x16 square of queries walks the squares of
    the 3x3 blocks around its own block.  Divisible grids, grids neither 16 nor the block side
    divides, a block larger than the grid (dense attention), and the running-maximum path (gain 14)."""
    monkeypatch.setenv("NSATTN_KERNEL", "block")
    q, k, v = synth.small_case(69, 1, 2, 64, gh, gw, "bf16")
    q = synth.round_to_bf16(q * gain)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, block) == "attn_block16_kernel"
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, 0.125, want_cls=True)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    ref = oracle.ns_attn(q, k, v, gh, gw, block, 0.125)
    assert_attn_close(to_np(out), ref, "bf16", "block kernel, %dx%d blocks on %dx%d" % (block, block, gh, gw))
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, 0.125, want_logits=True)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=2e-5 * gain)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=2e-5 * gain)


@pytest.mark.parametrize("gh,gw,block,gain", [(16, 16, 2, 1.0), (16, 24, 4, 1.0), (20, 27, 2, 1.0), (43, 30, 4, 1.0),
                                              (64, 64, 2, 1.0), (9, 9, 4, 1.0), (1, 1, 2, 1.0), (24, 16, 4, 14.0),
                                              (13, 40, 2, 14.0)])
def test_sweep_with_4x4_and_2x2_blocks(nb, monkeypatch, gh, gw, block, gain):
    """Blocks of side 4 and 2 on the sweep kernel's 8x8 tiles: pairs whose blocks are not neighbours
    are masked inside the tiles.  Also on grids that 8 (and the block side) does not divide, and
    through the running-maximum path (gain 14)."""
    monkeypatch.setenv("NSATTN_KERNEL", "sweep")
    q, k, v = synth.small_case(68, 2, 3, 64, gh, gw, "bf16")
    q = synth.round_to_bf16(q * gain)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    assert nb.ns_attn_patch_kernel_name(dq, gh, gw, block) == "attn_sweep_kernel"
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, 0.125, want_cls=True)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    ref = oracle.ns_attn(q, k, v, gh, gw, block, 0.125)
    assert_attn_close(to_np(out), ref, "bf16", "sweep, %dx%d blocks on %dx%d" % (block, block, gh, gw))
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, 0.125, want_logits=True)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=2e-5 * gain)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=2e-5 * gain)


def test_invalid_call_launches_nothing(nb):
    q = torch.zeros((1, 1, 65, 64), dtype=torch.bfloat16, device="cuda")
    out = torch.full_like(q, 7.0)
    with pytest.raises(nb.NsError) as e:
        nb.ns_attn_forward(q, q.clone(), q.clone(), 8, 9, 4, out=out)      # tokens != 1 + 72
    assert e.value.code == nb.NS_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("variant", ["mfma", "persist", "sweep", "block"])
@pytest.mark.parametrize("gh,gw,block", [(24, 40, 8), (8, 8, 8), (32, 32, 16), (48, 48, 8), (64, 64, 8), (96, 64, 16), (16, 72, 8), (40, 8, 8)])
def test_persistent_kernel_variant(nb, gh, gw, block, variant, monkeypatch):
    # the persistent-wave kernels compute the same function (grids too small for them fall back)
    monkeypatch.setenv("NSATTN_KERNEL", variant)
    run_case(nb, 303, 2, 5, gh, gw, block, "bf16")


@pytest.mark.parametrize("variant", ["mfma", "persist", "sweep", "block"])
def test_persistent_kernel_variant_overflow_fallback(nb, variant, monkeypatch):
    monkeypatch.setenv("NSATTN_KERNEL", variant)
    q, k, v = synth.small_case(7, 1, 2, 64, 16, 16, "bf16")
    q = synth.round_to_bf16(q * 12.0)
    ref = oracle.ns_attn(q, k, v, 16, 16, 8, 1.0)
    out = nb.ns_attn_forward(*(to_dev(a, "bf16") for a in (q, k, v)), 16, 16, 8, 1.0)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    assert_attn_close(to_np(out), ref, "bf16", "large logits, persistent kernel")


@pytest.mark.parametrize("variant", ["mfma", "persist", "sweep", "block"])
def test_persistent_kernel_partial_overflow(nb, variant, monkeypatch):
    """Only some query tiles overflow the fixed exponent reference: those are redone, the others not."""
    monkeypatch.setenv("NSATTN_KERNEL", variant)
    q, k, v = synth.small_case(11, 1, 3, 64, 32, 32, "bf16")
    q[:, :, 1 + 5 * 32:1 + 9 * 32] *= 14.0          # a band of grid rows with large logits
    q = synth.round_to_bf16(q)
    ref = oracle.ns_attn(q, k, v, 32, 32, 8, 1.0)
    out = nb.ns_attn_forward(*(to_dev(a, "bf16") for a in (q, k, v)), 32, 32, 8, 1.0)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    assert_attn_close(to_np(out), ref, "bf16", "partly large logits, persistent kernel")


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        block = int(rng.choice([2, 4, 8, 8, 8, 16, 16, 3, 5, 7, 12]))
        gh, gw = int(rng.integers(1, 72)), int(rng.integers(1, 72))
        force = str(rng.choice(["auto", "sweep", "block", "lists", "generic"]))
        cases.append((i, gh, gw, block, int(rng.integers(1, 3)), int(rng.integers(1, 4)), force,
                      float(rng.choice([1.0, 1.0, 1.0, 10.0])), float(rng.choice([0.125, 0.3, 0.05]))))
    return cases


@pytest.mark.parametrize("i,gh,gw,block,B,H,force,gain,scale", _random_cases(48, 2024))
def test_random_shapes_against_the_oracle(nb, monkeypatch, i, gh, gw, block, B, H, force, gain, scale):
    """Seeded random grids, block sides, batch and head counts, with a kernel forced at random (a forced
    kernel that does not take the problem falls back to the automatic choice): every output row,
    the global query's logits and log-sum-exp against the oracle."""
    if force != "auto":
        monkeypatch.setenv("NSATTN_KERNEL", force)
    q, k, v = synth.small_case(5000 + i, B, H, 64, gh, gw, "bf16")
    q = synth.round_to_bf16(q * gain)
    dq, dk, dv = (to_dev(a, "bf16") for a in (q, k, v))
    print("case %d: grid %dx%d block %d B=%d H=%d force=%s gain=%g scale=%g -> %s" % (
        i, gh, gw, block, B, H, force, gain, scale, nb.ns_attn_patch_kernel_name(dq, gh, gw, block, scale)), flush=True)
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, gh, gw, block, scale, want_cls=True)
    torch.cuda.synchronize()
    assert np.isfinite(to_np(out)).all()
    ref = oracle.ns_attn(q, k, v, gh, gw, block, scale)
    assert_attn_close(to_np(out), ref, "bf16", "random case %d" % i)
    _, ref_logits, ref_lse = oracle.cls_scores(q, k, scale, want_logits=True)
    tol = 2e-5 * gain * max(1.0, scale / 0.125)
    np.testing.assert_allclose(to_np(logits), ref_logits, rtol=0, atol=tol)
    np.testing.assert_allclose(to_np(lse), ref_lse, rtol=0, atol=tol)
