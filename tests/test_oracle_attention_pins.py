"""Pins for the CPU oracle's attention: each test checks oracle/ns_oracle.c against
something that is not the oracle -- a dense masked attention whose mask is written on
pixel coordinates, a library attention routine, closed forms and invariants of the
pattern described in the paper's "Memory-Efficiency Optimization" section."""
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2601_12150_amd import synth

PATCH = 16  # pixels per patch side; only used to phrase the mask in pixel space


def dense_masked_attention(q, k, v, grid_h, grid_w, block, scale, radius=1, kept=None):
    """Textbook dense softmax attention with -inf on masked logits.  The mask is phrased on
    patch *pixel* positions: two patches may interact when the pixel windows of side
    block*PATCH they fall in are at most `radius` windows apart in x and in y."""
    B, H, T, D = q.shape
    n = grid_h * grid_w if kept is None else len(kept)
    idx = np.arange(grid_h * grid_w) if kept is None else np.asarray(kept)
    y_px = (idx // grid_w) * PATCH + PATCH // 2          # patch centre, pixels
    x_px = (idx % grid_w) * PATCH + PATCH // 2
    wy = y_px // (block * PATCH)
    wx = x_px // (block * PATCH)
    mask = np.ones((T, T), dtype=bool)
    near = (np.abs(wy[:, None] - wy[None, :]) <= radius) & (np.abs(wx[:, None] - wx[None, :]) <= radius)
    mask[1:, 1:] = near
    assert T == n + 1
    s = np.einsum("bhid,bhjd->bhij", q.astype(np.float64), k.astype(np.float64)) * scale
    s = np.where(mask, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=-1, keepdims=True)
    return np.einsum("bhij,bhjd->bhid", p, v.astype(np.float64)), p, mask


@pytest.mark.parametrize("gh,gw,block", [(4, 4, 1), (6, 6, 2), (9, 9, 3), (12, 12, 4), (8, 8, 4),
                                         (4, 4, 4), (12, 12, 3), (6, 10, 2), (7, 5, 2), (10, 9, 4)])
def test_matches_dense_masked_reference(gh, gw, block):
    q, k, v = synth.small_case(11, 2, 3, 8, gh, gw)
    ref, pref, _ = dense_masked_attention(q, k, v, gh, gw, block, 0.35)
    out, prob = oracle.ns_attn(q, k, v, gh, gw, block, 0.35, want_prob=True)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    np.testing.assert_allclose(prob, pref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("gh,gw,block,radius", [(10, 10, 2, 2), (8, 8, 2, 0), (9, 6, 1, 3)])
def test_other_radii_match_dense_masked_reference(gh, gw, block, radius):
    q, k, v = synth.small_case(5, 1, 2, 4, gh, gw)
    ref, _, _ = dense_masked_attention(q, k, v, gh, gw, block, 0.5, radius=radius)
    out = oracle.ns_attn(q, k, v, gh, gw, block, 0.5, radius=radius)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("g,block", [(8, 4), (8, 8), (6, 3), (5, 16)])
def test_equals_library_dense_attention_when_neighbourhood_covers_grid(g, block):
    # at most two blocks per side: every block neighbours every other block
    q, k, v = synth.small_case(3, 2, 4, 16, g, g)
    out = oracle.ns_attn(q, k, v, g, g, block, 0.25)
    tq, tk, tv = (torch.from_numpy(a).double() for a in (q, k, v))
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=0.25).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("gh,gw,block", [(28, 28, 7), (64, 64, 8), (12, 20, 4), (9, 9, 3)])
def test_pair_count_closed_form(gh, gw, block):
    nbh, nbw = gh // block, gw // block
    N = gh * gw
    def span(nb):  # sum over blocks of the number of neighbours along one axis
        return 3 * nb - 2 if nb > 1 else 1
    expect = span(nbh) * span(nbw) * block ** 4 + 2 * N + 1
    assert oracle.count_pairs(1 + N, gw, block) == expect


def test_pair_counts_of_the_workload_grids():
    """tests/golden/pair_counts.txt: counts fixed by the pattern for the measured grids."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "pair_counts.txt")
    rows = [line.split() for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) >= 3
    for tokens, grid_w, block, pairs in rows:
        assert oracle.count_pairs(int(tokens), int(grid_w), int(block)) == int(pairs)


def test_locality_keys_outside_the_neighbourhood_do_not_matter():
    g, block = 12, 3
    q, k, v = synth.small_case(7, 1, 2, 8, g, g)
    out = oracle.ns_attn(q, k, v, g, g, block, 0.3)
    # query patch (4,4) lives in block (1,1): neighbourhood = blocks 0..2 -> rows/cols 0..8
    r, c = np.divmod(np.arange(g * g), g)
    outside = 1 + np.flatnonzero((r >= 9) | (c >= 9))
    k2, v2 = k.copy(), v.copy()
    k2[:, :, outside] += 5.0
    v2[:, :, outside] -= 3.0
    out2 = oracle.ns_attn(q, k2, v2, g, g, block, 0.3)
    qi = 1 + 4 * g + 4
    assert np.array_equal(out[:, :, qi], out2[:, :, qi])
    # a query in block (3,3) does see some of the changed keys
    qj = 1 + 10 * g + 10
    assert not np.allclose(out[:, :, qj], out2[:, :, qj])
    # and perturbing a key just inside the neighbourhood of (4,4) changes it
    k3 = k.copy()
    k3[:, :, 1 + 8 * g + 8] += 5.0
    out3 = oracle.ns_attn(q, k3, v, g, g, block, 0.3)
    assert not np.allclose(out[:, :, qi], out3[:, :, qi])


@pytest.mark.parametrize("op", ["fliplr", "flipud", "transpose"])
def test_grid_symmetries_permute_the_output(op):
    g, block = 8, 2
    q, k, v = synth.small_case(9, 1, 2, 8, g, g)
    grid_idx = np.arange(g * g).reshape(g, g)
    perm_grid = {"fliplr": grid_idx[:, ::-1], "flipud": grid_idx[::-1], "transpose": grid_idx.T}[op]
    perm = np.concatenate([[0], 1 + perm_grid.reshape(-1)])
    out = oracle.ns_attn(q, k, v, g, g, block, 0.3)
    outp = oracle.ns_attn(q[:, :, perm], k[:, :, perm], v[:, :, perm], g, g, block, 0.3)
    np.testing.assert_allclose(outp, out[:, :, perm], rtol=0, atol=1e-13)


def test_zero_queries_give_the_mean_of_allowed_values():
    g, block = 9, 3
    q, k, v = synth.small_case(13, 1, 2, 4, g, g)
    q[:] = 0
    out = oracle.ns_attn(q, k, v, g, g, block, 1.0)
    _, _, mask = dense_masked_attention(q, k, v, g, g, block, 1.0)
    v64 = v.astype(np.float64)
    for i in (0, 1, 1 + 4 * g + 4, 1 + 8 * g + 8, 1 + 3 * g):
        expect = v64[:, :, mask[i]].mean(axis=2)
        np.testing.assert_allclose(out[:, :, i], expect, rtol=0, atol=1e-13)
    # corner query: CLS + 2x2 blocks of 9 patches
    assert mask[1].sum() == 1 + 4 * 9 and mask[1 + 4 * g + 4].sum() == 1 + 81


def test_constant_values_are_reproduced():
    g, block = 8, 2
    q, k, v = synth.small_case(17, 2, 2, 8, g, g)
    v[:] = np.linspace(-1, 1, 8, dtype=np.float32)
    out = oracle.ns_attn(q, k, v, g, g, block, 0.7)
    np.testing.assert_allclose(out, np.broadcast_to(v.astype(np.float64), out.shape), atol=1e-14)


def test_one_dominant_logit_selects_that_value_row():
    g, block = 8, 2
    q, k, v = synth.small_case(19, 1, 1, 8, g, g)
    qi, kj = 1 + 3 * g + 3, 1 + 2 * g + 4     # blocks (1,1) and (1,2): neighbours
    k[0, 0, kj] = 200.0 * q[0, 0, qi]
    out = oracle.ns_attn(q, k, v, g, g, block, 1.0)
    np.testing.assert_allclose(out[0, 0, qi], v[0, 0, kj].astype(np.float64), atol=1e-9)
    # the same huge key is invisible to a far query (block (3,0)); its row stays a mixture
    far = 1 + 7 * g + 0
    assert np.abs(out[0, 0, far] - v[0, 0, kj]).max() > 1e-3


def test_pruned_sequence_uses_original_grid_positions():
    # attention on a kept subset == dense masked attention restricted to those tokens
    g, block = 12, 3
    rng = np.random.default_rng(5)
    kept = np.sort(rng.choice(g * g, size=70, replace=False))
    # empty one whole block and leave one patch alone in its neighbourhood
    r, c = np.divmod(kept, g)
    kept = kept[~((r // block == 0) & (c // block == 0))]
    q, k, v = synth.small_case(23, 2, 2, 8, 1, len(kept))
    coords = np.broadcast_to(synth.raster_coords(g, g)[kept], (2, len(kept)))
    ref, _, _ = dense_masked_attention(q, k, v, g, g, block, 0.4, kept=kept)
    out = oracle.ns_attn(q, k, v, g, g, block, 0.4, coords=coords)
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


def test_row_subset_equals_full_run():
    g, block = 8, 2
    q, k, v = synth.small_case(29, 1, 2, 8, g, g)
    rows = np.array([0, 5, 33, 64], dtype=np.int32)
    full = oracle.ns_attn(q, k, v, g, g, block, 0.3)
    sub = oracle.ns_attn(q, k, v, g, g, block, 0.3, rows=rows)
    assert np.array_equal(sub, full[:, :, rows])


def test_several_global_tokens():
    g, block, G = 6, 2, 3
    q, k, v = synth.small_case(31, 1, 2, 8, g, g, n_global=G)
    out = oracle.ns_attn(q, k, v, g, g, block, 0.3, n_global=G)
    T = G + g * g
    r, c = np.divmod(np.arange(g * g), g)
    near = (np.abs(r[:, None] // block - r[None, :] // block) <= 1) & \
           (np.abs(c[:, None] // block - c[None, :] // block) <= 1)
    mask = np.ones((T, T), dtype=bool)
    mask[G:, G:] = near
    s = np.einsum("bhid,bhjd->bhij", q.astype(np.float64), k.astype(np.float64)) * 0.3
    s = np.where(mask, s, -np.inf)
    p = np.exp(s - s.max(-1, keepdims=True))
    p /= p.sum(-1, keepdims=True)
    np.testing.assert_allclose(out, p @ v.astype(np.float64), atol=1e-12)
