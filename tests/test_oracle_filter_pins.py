"""Pins for the oracle's scoring, ranking and compaction (paper, "Time-Efficiency
Optimization": score from the global token's attention weights, rank, discard the
lowest, shorten the sequence)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2601_12150_amd import synth


def softmax64(x):
    x = x - x.max(axis=-1, keepdims=True)
    e = np.exp(x)
    return e / e.sum(axis=-1, keepdims=True)


def test_scores_are_row_zero_of_dense_attention_averaged_over_heads():
    g = 7
    q, k, v = synth.small_case(41, 2, 5, 8, g, g)
    s = np.einsum("bhd,bhjd->bhj", q[:, :, 0].astype(np.float64), k.astype(np.float64)) * 0.3
    p = softmax64(s)
    expect = p[:, :, 1:].mean(axis=1)
    got, logits, lse = oracle.cls_scores(q, k, 0.3, want_logits=True)
    np.testing.assert_allclose(got, expect, rtol=0, atol=1e-15)
    np.testing.assert_allclose(logits, s, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, np.log(np.exp(s).sum(-1)), rtol=0, atol=1e-12)
    # the same numbers as the attention oracle's own CLS row
    _, prob = oracle.ns_attn(q, k, v, g, g, 2, 0.3, rows=np.array([0], dtype=np.int32), want_prob=True)
    np.testing.assert_allclose(got, prob[:, :, 0, 1:].mean(axis=1), rtol=0, atol=1e-15)


def test_score_sum_identity_and_zero_query():
    g = 6
    q, k, _ = synth.small_case(43, 1, 4, 8, g, g)
    a = oracle.cls_scores(q, k, 0.5)
    s = np.einsum("bhd,bhjd->bhj", q[:, :, 0].astype(np.float64), k.astype(np.float64)) * 0.5
    p00 = softmax64(s)[:, :, 0]
    np.testing.assert_allclose(a.sum(axis=1), 1.0 - p00.mean(axis=1), atol=1e-14)
    q[:] = 0
    a0 = oracle.cls_scores(q, k, 0.5)
    np.testing.assert_allclose(a0, 1.0 / (1 + g * g), atol=1e-16)


def test_scores_with_several_global_rows_average_those_rows():
    g, G = 5, 2
    q, k, _ = synth.small_case(47, 1, 3, 8, g, g, n_global=G)
    s = np.einsum("bhgd,bhjd->bhgj", q[:, :, :G].astype(np.float64), k.astype(np.float64)) * 0.4
    expect = softmax64(s)[..., G:].mean(axis=(1, 2))
    np.testing.assert_allclose(oracle.cls_scores(q, k, 0.4, n_global=G), expect, atol=1e-15)


def brute_force_topk(scores, k):
    """All k-subsets of a tiny score vector: the best one under (score desc, index asc)."""
    n = len(scores)
    best = None
    for sub in itertools.combinations(range(n), k):
        rest = [j for j in range(n) if j not in sub]
        ok = all((scores[i] > scores[j]) or (scores[i] == scores[j] and i < j)
                 for i in sub for j in rest)
        if ok:
            assert best is None, "selection must be unique"
            best = sub
    return np.array(best, dtype=np.int32)


@pytest.mark.parametrize("seed", range(6))
def test_topk_against_subset_enumeration(seed):
    rng = np.random.default_rng(seed)
    n = 9
    s = rng.integers(0, 4, size=n).astype(np.float32)      # many exact ties
    for k in (1, 3, 4, 8, 9):
        got = oracle.topk(s[None], k)[0]
        assert np.array_equal(got, brute_force_topk(s, k))


def test_topk_invariants_and_special_cases():
    rng = np.random.default_rng(3)
    s = rng.random((3, 1000)).astype(np.float32)
    k = 377
    kept = oracle.topk(s, k)
    ref = np.sort(np.argsort(-s, axis=1, kind="stable")[:, :k], axis=1)
    assert np.array_equal(kept, ref)
    for b in range(3):
        assert np.all(np.diff(kept[b]) > 0)
        dropped = np.setdiff1d(np.arange(1000), kept[b])
        assert s[b, kept[b]].min() >= s[b, dropped].max()
    # all equal -> the first k indices; k = N -> identity; k = 1 -> argmax
    assert np.array_equal(oracle.topk(np.ones((1, 50), np.float32), 20)[0], np.arange(20))
    assert np.array_equal(oracle.topk(s, 1000)[1], np.arange(1000))
    assert np.array_equal(oracle.topk(s, 1)[:, 0], s.argmax(axis=1))
    # negative, zero and denormal scores are ordered as numbers, not as bit patterns
    t = np.array([[-1.0, 0.0, -0.0, 1e-40, -2.5, 3.0]], np.float32)
    assert np.array_equal(oracle.topk(t, 3)[0], [1, 3, 5])


def test_gather_is_a_bit_copy_with_cls_first():
    rng = np.random.default_rng(1)
    x = rng.integers(0, 2 ** 16, size=(2, 1 + 30, 12), dtype=np.uint16)   # raw bf16 bit patterns
    kept = np.array([[0, 3, 4, 29], [1, 2, 10, 11]], dtype=np.int32)
    y = oracle.gather(x, kept)
    assert y.shape == (2, 5, 12)
    for b in range(2):
        assert np.array_equal(y[b, 0], x[b, 0])
        for t in range(4):
            assert np.array_equal(y[b, 1 + t], x[b, 1 + kept[b, t]])
    with pytest.raises(ValueError):
        oracle.gather(x, np.array([[0, 30], [0, 1]], dtype=np.int32))


def test_gather_with_several_global_tokens_hand_built():
    """oracle.gather with G > 1: the G leading rows stay, then rows G + kept[b, t]; expected rows
    written out by hand (no formula shared with the oracle)."""
    B, G, N, C = 2, 3, 5, 4
    x = (np.arange(B * (G + N) * C, dtype=np.float32).reshape(B, G + N, C) * 7 % 31).astype(np.float32)
    kept = np.array([[0, 2, 4], [1, 2, 3]], dtype=np.int32)
    y = oracle.gather(x, kept, n_global=G)
    assert y.shape == (B, G + 3, C)
    want0 = [x[0, 0], x[0, 1], x[0, 2], x[0, 3], x[0, 5], x[0, 7]]        # globals 0..2, patches 0, 2, 4 -> rows 3, 5, 7
    want1 = [x[1, 0], x[1, 1], x[1, 2], x[1, 4], x[1, 5], x[1, 6]]        # patches 1, 2, 3 -> rows 4, 5, 6
    assert np.array_equal(y[0], np.stack(want0)) and np.array_equal(y[1], np.stack(want1))
    # bit copy also of patterns that are not numbers
    xb = np.full((1, G + N, 2), 0x7FC1, dtype=np.uint16)
    xb[0, :, 1] = np.arange(G + N, dtype=np.uint16) + 0xFF80
    yb = oracle.gather(xb, np.array([[4]], dtype=np.int32), n_global=G)
    assert np.array_equal(yb[0, :, 1], np.array([0xFF80, 0xFF81, 0xFF82, 0xFF87], dtype=np.uint16))
    # G = 1 on the same data keeps one leading row and shifts the patches by one
    y1 = oracle.gather(x, kept, n_global=1)
    assert np.array_equal(y1[0], np.stack([x[0, 0], x[0, 1], x[0, 3], x[0, 5]]))
    # an index beyond the patches of the G > 1 layout is refused
    import pytest
    with pytest.raises(ValueError):
        oracle.gather(x, np.array([[0, 1, 5], [0, 1, 2]], dtype=np.int32), n_global=G)
