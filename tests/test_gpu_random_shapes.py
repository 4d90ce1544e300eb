"""Seeded random sweeps through the C ABI against the oracle: shapes, block sides, kernel choices,
numbers of global tokens, pruned subsets and logit gains drawn at random within the documented
limits (attention + scores), and row lengths, keep counts and score distributions (selection)."""
import random

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


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_attention_and_scores_on_random_problems(nb, monkeypatch, seed):
    rng = random.Random(seed)
    for it in range(40):
        force = rng.choice(["", "", "sweep", "block", "persist", "mfma", "lists", "generic"])
        block = rng.choice([2, 4, 8, 8, 8, 16, 16, 32, 3, 5, 7, 12])
        gh, gw = rng.randint(1, 70), rng.randint(1, 70)
        if rng.random() < 0.4:     # grids the block side divides
            gh, gw = block * rng.randint(1, max(1, 64 // block)), block * rng.randint(1, max(1, 64 // block))
        B, H = rng.randint(1, 3), rng.randint(1, 4)
        G = rng.choice([1, 1, 1, 2, 3, 5, 8, 9])
        dtype = "bf16" if force != "generic" or rng.random() < 0.5 else "f32"
        gain = rng.choice([1.0, 1.0, 1.0, 6.0, 14.0])
        if force:
            monkeypatch.setenv("NSATTN_KERNEL", force)
        else:
            monkeypatch.delenv("NSATTN_KERNEL", raising=False)
        q, k, v = synth.small_case(1000 * seed + it, B, H, 64, gh, gw, dtype, n_global=G)
        if gain != 1.0:
            q = synth.round_to_bf16(q * np.float32(gain)) if dtype == "bf16" else q * np.float32(gain)
        coords = None
        if rng.random() < 0.25 and gh * gw > 4:
            kept = np.sort(np.random.default_rng(it).choice(gh * gw, size=rng.randint(1, gh * gw), replace=False))
            sel = np.concatenate([np.arange(G), G + kept])
            q, k, v = (np.ascontiguousarray(a[:, :, sel]) for a in (q, k, v))
            coords = np.tile(synth.raster_coords(gh, gw)[kept], (B, 1))
        what = "seed %d case %d: kernel %r B=%d H=%d grid %dx%d block %d G=%d %s gain %g pruned to %s" % (
            seed, it, force, B, H, gh, gw, block, G, dtype, gain, None if coords is None else coords.shape[1])
        print(what, flush=True)
        ref = oracle.ns_attn(q, k, v, gh, gw, block, 0.125, coords=coords, n_global=G)
        dq, dk, dv = (to_dev(a, dtype) for a in (q, k, v))
        dc = None if coords is None else torch.from_numpy(coords).cuda()
        out, logits, lse, scores = nb.ns_attn_forward_scores(dq, dk, dv, gh, gw, block, 0.125, coords=dc, n_global=G)
        torch.cuda.synchronize()
        assert_attn_close(to_np(out), ref, dtype, what)
        np.testing.assert_allclose(to_np(scores), oracle.cls_scores(q, k, 0.125, n_global=G), rtol=1e-4, atol=1e-9, err_msg=what)


def test_selection_on_random_rows(nb):
    rng = random.Random(7)
    for it in range(90):
        B = rng.randint(1, 4)
        if it % 3:
            N = rng.choice([rng.randint(1, 5000), rng.randint(1, 40000), rng.randint(30000, 140000)])
        else:
            N = rng.choice([1024, 4096, 4097, 8192, 16384, 16385, 32768, 32769, 65536])
        k = rng.choice([1, N, rng.randint(1, N), max(1, N * 6 // 10)])
        kind = rng.choice(["uniform", "ties", "cluster", "signed", "const"])
        r = np.random.default_rng(it)
        if kind == "uniform":
            s = r.random((B, N)).astype(np.float32)
        elif kind == "ties":
            s = r.integers(0, rng.choice([2, 5, 50]), size=(B, N)).astype(np.float32)
        elif kind == "cluster":
            s = (1e-4 * (1 + 1e-3 * r.standard_normal((B, N)))).astype(np.float32)
            s[:, : N // 3] = (r.random((B, N // 3)) * 2e-4).astype(np.float32)
        elif kind == "signed":
            s = r.standard_normal((B, N)).astype(np.float32)
            s[:, ::5] = 0.0
            s[:, 1::7] = -0.0
        else:
            s = np.full((B, N), 0.5, np.float32)
        coords = r.integers(0, 2 ** 31 - 1, size=(B, N), dtype=np.int32)
        what = "case %d: B=%d N=%d k=%d %s" % (it, B, N, k, kind)
        print(what, flush=True)
        ref = oracle.topk(s, k)
        kept, _, cout = nb.topk_filter(torch.from_numpy(s).cuda(), k, coords=torch.from_numpy(coords).cuda())
        torch.cuda.synchronize()
        assert np.array_equal(kept.cpu().numpy(), ref), what
        assert np.array_equal(cout.cpu().numpy(), np.take_along_axis(coords, ref.astype(np.int64), axis=1)), what
