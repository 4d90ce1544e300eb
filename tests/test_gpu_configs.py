"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times:
outputs of sampled query rows (the oracle computes them one by one), scores and kept sets."""
import numpy as np
import pytest
import torch

import oracle
from paper_2601_12150_amd import synth
from _util import assert_attn_close, assert_kept_sets_match, to_dev, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def sample_rows(cfg, n, seed):
    """CLS, the four grid corners, edge and interior patches, then random ones."""
    g = cfg.grid
    fixed = [0, 1, g, 1 + (g - 1) * g, g * g, 1 + g // 2, 1 + (g // 2) * g, 1 + (g // 2) * g + g // 2,
             1 + (cfg.block - 1) * g + cfg.block - 1, 1 + cfg.block * g + cfg.block]
    rng = np.random.default_rng(seed)
    rest = rng.choice(np.arange(1, cfg.tokens), size=n - len(fixed), replace=False)
    return np.unique(np.concatenate([fixed, rest])).astype(np.int32)


@pytest.mark.parametrize("cfg_id,n_rows", [(1, 785), (2, 160), (3, 96), (4, 40),
                                           (11, 96), (12, 48), (13, 40), (14, 24), (15, 64)])
def test_config_pipeline(nb, cfg_id, n_rows):
    cfg = synth.CONFIGS[cfg_id]
    print("config", cfg.name, flush=True)
    q, k, v, info = synth.make_qkv(cfg)
    dq, dk, dv = (to_dev(a, cfg.dtype) for a in (q, k, v))
    out, logits, lse = nb.ns_attn_forward(dq, dk, dv, cfg.grid, cfg.grid, cfg.block, cfg.scale, want_cls=True)
    torch.cuda.synchronize()
    rows = np.arange(cfg.tokens, dtype=np.int32) if n_rows >= cfg.tokens else sample_rows(cfg, n_rows, cfg.seed)
    ref = oracle.ns_attn(q, k, v, cfg.grid, cfg.grid, cfg.block, cfg.scale, rows=rows)
    got = to_np(out[:, :, torch.from_numpy(rows.astype(np.int64)).cuda()])
    assert_attn_close(got, ref, cfg.dtype, cfg.name)
    # property that holds at any size: every output row is a convex combination of value rows
    vmin = dv.float().amin(dim=2, keepdim=True) - 1e-2
    vmax = dv.float().amax(dim=2, keepdim=True) + 1e-2
    o = out.float()
    assert bool(((o >= vmin) & (o <= vmax)).all()) and bool(torch.isfinite(o).all())

    # scores: standalone and fused agree with the oracle; kept sets match outside the tie band
    ref_scores = oracle.cls_scores(q, k, cfg.scale)
    s1 = nb.cls_scores(dq, dk, cfg.scale)
    s2 = nb.cls_scores_from_logits(logits, lse)
    torch.cuda.synchronize()
    np.testing.assert_allclose(to_np(s1), ref_scores, rtol=5e-5, atol=1e-10)
    np.testing.assert_allclose(to_np(s2), ref_scores, rtol=5e-5, atol=1e-10)
    ref_kept = oracle.topk(ref_scores.astype(np.float32), cfg.k)
    x = to_dev(synth.make_tokens(cfg), cfg.dtype)
    kept, y, _ = nb.topk_filter(s1, cfg.k, x=x)
    torch.cuda.synchronize()
    kept_np = kept.cpu().numpy()
    assert_kept_sets_match(kept_np, ref_kept, ref_scores, cfg.k)
    # selection is bit-exact on the scores the GPU itself produced
    assert np.array_equal(kept_np, oracle.topk(s1.cpu().numpy(), cfg.k))
    # compaction is a bit copy of the chosen rows
    idx = torch.cat([torch.zeros((cfg.batch, 1), dtype=torch.int64, device="cuda"), kept.long() + 1], dim=1)
    expect = torch.gather(x, 1, idx[:, :, None].expand(-1, -1, x.shape[2]))
    assert torch.equal(y, expect)
    if "background" in info:
        bg = info["background"].reshape(cfg.batch, -1)
        dropped = np.ones_like(bg)
        np.put_along_axis(dropped, kept_np.astype(np.int64), False, axis=1)
        print("background fraction %.3f, among dropped tokens %.3f" % (bg.mean(), bg[dropped].mean()), flush=True)
