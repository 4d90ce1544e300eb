"""GPU parity: cls_scores, cls_scores_from_logits and topk_filter against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_12150_amd import synth
from _util import assert_kept_sets_match, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


@pytest.mark.parametrize("dtype,g,B,H", [("bf16", 24, 2, 16), ("f32", 28, 1, 16), ("bf16", 45, 3, 5),
                                         ("f32", 7, 2, 3), ("bf16", 1, 1, 1)])
def test_cls_scores_standalone_and_fused(nb, dtype, g, B, H):
    q, k, v = synth.small_case(61, B, H, 64, g, g, dtype)
    ref = oracle.cls_scores(q, k, 0.125)
    dq, dk, dv = (to_dev(a, dtype) for a in (q, k, v))
    got = nb.cls_scores(dq, dk, 0.125)
    # scores are O(1/T); fp32 arithmetic on exact inputs: relative error ~1e-6
    np.testing.assert_allclose(to_np(got), ref, rtol=2e-5, atol=1e-9)
    # the same numbers from the attention call's by-products
    _, logits, lse = nb.ns_attn_forward(dq, dk, dv, g, g, 4, 0.125, want_cls=True)
    fused = nb.cls_scores_from_logits(logits, lse)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_np(fused), ref, rtol=2e-5, atol=1e-9)


@pytest.mark.parametrize("dtype,g,block,B,H,G,force", [
    ("bf16", 24, 8, 2, 16, 1, "sweep"), ("bf16", 48, 16, 1, 4, 1, "block"), ("bf16", 30, 5, 2, 3, 1, None),
    ("f32", 28, 7, 1, 16, 1, None), ("bf16", 37, 8, 1, 2, 1, "sweep"), ("bf16", 20, 4, 2, 3, 3, None),
    ("bf16", 1, 8, 1, 1, 1, None)])
def test_attention_and_scores_in_one_call(nb, monkeypatch, dtype, g, block, B, H, G, force):
    """ns_attn_forward_scores: the attention outputs and by-products are bit-equal to
    ns_attn_forward's, and the scores (merged and computed in one launch) match the oracle."""
    if force:
        monkeypatch.setenv("NSATTN_KERNEL", force)
    if G == 1:
        q, k, v = synth.small_case(62, B, H, 64, g, g, dtype)
    else:
        rng = np.random.default_rng(62)
        shape = (B, H, G + g * g, 64)
        q, k, v = (synth.round_to_bf16(rng.standard_normal(shape).astype(np.float32)) for _ in range(3))
    ref = oracle.cls_scores(q, k, 0.125, n_global=G) if G > 1 else oracle.cls_scores(q, k, 0.125)
    dq, dk, dv = (to_dev(a, dtype) for a in (q, k, v))
    out, logits, lse, scores = nb.ns_attn_forward_scores(dq, dk, dv, g, g, block, 0.125, n_global=G)
    out2, logits2, lse2 = nb.ns_attn_forward(dq, dk, dv, g, g, block, 0.125, want_cls=True, n_global=G)
    torch.cuda.synchronize()
    assert torch.equal(out, out2) and torch.equal(logits, logits2) and torch.equal(lse, lse2)
    np.testing.assert_allclose(to_np(scores), ref, rtol=2e-5, atol=1e-9)


def topk_case(nb, scores, k):
    ref = oracle.topk(scores, k)
    kept, _, _ = nb.topk_filter(torch.from_numpy(scores).cuda(), k)
    torch.cuda.synchronize()
    assert np.array_equal(kept.cpu().numpy(), ref)


@pytest.mark.parametrize("N,k", [(1, 1), (7, 3), (64, 64), (1000, 377), (1024, 1), (4096, 2458),
                                 (16384, 9831), (65536, 26215), (70001, 35000)])
def test_topk_random_scores_bit_exact(nb, N, k):
    rng = np.random.default_rng(N + k)
    topk_case(nb, rng.random((3, N)).astype(np.float32), k)


def test_topk_ties_signs_and_clusters(nb):
    rng = np.random.default_rng(9)
    # heavy exact ties: the lower index must win
    topk_case(nb, rng.integers(0, 5, size=(2, 5000)).astype(np.float32), 1234)
    # all equal
    topk_case(nb, np.full((2, 3000), 0.25, np.float32), 1000)
    # negative, zero, minus zero, denormals, infinities
    s = rng.standard_normal((2, 4000)).astype(np.float32)
    s[:, ::7] = 0.0
    s[:, 3::7] = -0.0
    s[:, 5::11] = 1e-40
    s[0, 17] = np.inf
    s[1, 23] = -np.inf
    for k in (1, 500, 2000, 3999, 4000):
        topk_case(nb, s, k)
    # clustered like the background tokens: most keys share their leading digits
    c = (1e-4 * (1.0 + 1e-3 * rng.standard_normal((2, 16384)))).astype(np.float32)
    c[:, :6000] = rng.random((2, 6000)).astype(np.float32) * 2e-4
    topk_case(nb, c, 9831)


@pytest.mark.parametrize("N", [16385, 17408, 32768, 32769, 60025, 65536, 65537, 131072, 131073, 300000])
def test_topk_long_rows(nb, N):
    """Rows of up to 32768 scores are selected by one workgroup per image with up to 32 keys per
    thread, longer ones by several workgroups per image (digit histograms exchanged between
    launches): random, tied, clustered and signed scores, k from 1 to N, the coordinates compacted
    along."""
    rng = np.random.default_rng(N)
    topk_case(nb, rng.random((2, N)).astype(np.float32), (N * 6) // 10)
    topk_case(nb, rng.integers(0, 4, size=(2, N)).astype(np.float32), N // 3)          # heavy ties across chunks
    topk_case(nb, np.full((1, N), 0.5, np.float32), N // 2)                              # all equal
    c = (1e-5 * (1.0 + 1e-3 * rng.standard_normal((2, N)))).astype(np.float32)          # clustered
    c[:, : N // 3] = rng.random((2, N // 3)).astype(np.float32) * 2e-5
    topk_case(nb, c, (N * 6) // 10)
    s = rng.standard_normal((2, N)).astype(np.float32)
    s[:, ::7] = 0.0
    s[:, 3::7] = -0.0
    s[0, 17] = np.inf
    s[1, N - 1] = -np.inf
    for k in (1, 2, N // 2, N - 1, N):
        topk_case(nb, s, k)
    coords = rng.integers(0, 2 ** 31 - 1, size=(2, N), dtype=np.int32)
    kept, _, cout = nb.topk_filter(torch.from_numpy(c).cuda(), N // 5, coords=torch.from_numpy(coords).cuda())
    torch.cuda.synchronize()
    ref = oracle.topk(c, N // 5)
    assert np.array_equal(kept.cpu().numpy(), ref)
    assert np.array_equal(cout.cpu().numpy(), np.take_along_axis(coords, ref.astype(np.int64), axis=1))


def test_gather_and_coords_compaction_bit_exact(nb):
    rng = np.random.default_rng(4)
    B, N, C, k = 2, 500, 1024, 301
    scores = rng.random((B, N)).astype(np.float32)
    xbits = rng.integers(0, 2 ** 16, size=(B, 1 + N, C), dtype=np.uint16)     # arbitrary bf16 bit patterns
    x = torch.from_numpy(xbits.view(np.int16)).cuda().view(torch.bfloat16)
    coords = rng.integers(0, 2 ** 31 - 1, size=(B, N), dtype=np.int32)
    kept, y, cout = nb.topk_filter(torch.from_numpy(scores).cuda(), k, x=x, coords=torch.from_numpy(coords).cuda())
    torch.cuda.synchronize()
    ref_kept = oracle.topk(scores, k)
    assert np.array_equal(kept.cpu().numpy(), ref_kept)
    ybits = y.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(ybits, oracle.gather(xbits, ref_kept))
    assert np.array_equal(cout.cpu().numpy(), np.take_along_axis(coords, ref_kept.astype(np.int64), axis=1))
    # fp32 rows
    xf = rng.standard_normal((B, 1 + N, 68)).astype(np.float32)
    _, yf, _ = nb.topk_filter(torch.from_numpy(scores).cuda(), k, x=torch.from_numpy(xf).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(yf.cpu().numpy(), oracle.gather(xf, ref_kept))


def test_scores_to_kept_set_end_to_end(nb):
    g = 40
    q, k, v = synth.small_case(77, 2, 16, 64, g, g, "bf16")
    ref_scores = oracle.cls_scores(q, k, 0.125)
    kk = (g * g * 60 + 99) // 100
    ref_kept = oracle.topk(ref_scores.astype(np.float32), kk)
    got_scores = nb.cls_scores(to_dev(q, "bf16"), to_dev(k, "bf16"), 0.125)
    kept, _, _ = nb.topk_filter(got_scores, kk)
    torch.cuda.synchronize()
    assert_kept_sets_match(kept.cpu().numpy(), ref_kept, ref_scores, kk)
