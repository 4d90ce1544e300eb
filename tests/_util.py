"""Helpers shared by the GPU parity tests: tensor transfer and the parity bars."""
import numpy as np
import torch


def to_dev(x: np.ndarray, dtype: str) -> torch.Tensor:
    """float32 numpy array (values representable in dtype) -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)      # exact: the values are already bf16-representable
    return t.cuda()


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def assert_attn_close(gpu: np.ndarray, ref: np.ndarray, dtype: str, what: str = ""):
    """fp32: max-abs <= 1e-4.  bf16 storage with fp32 accumulation: element-wise
    |gpu - ref| <= 2e-2*|ref| + 2e-2*rms(ref) (pure relative error is unbounded near zero)."""
    err = np.abs(gpu - ref)
    if dtype == "f32":
        assert err.max() <= 1e-4, "%s max-abs error %.3g > 1e-4" % (what, err.max())
    else:
        rms = float(np.sqrt(np.mean(ref ** 2)))
        bound = 2e-2 * np.abs(ref) + 2e-2 * rms
        worst = float((err - bound).max())
        assert worst <= 0, "%s bf16 bound exceeded by %.3g (max err %.3g, rms %.3g)" % (
            what, worst, err.max(), rms)
        rel_l2 = float(np.sqrt((err ** 2).sum() / (ref ** 2).sum()))
        assert rel_l2 <= 1e-2, "%s relative L2 error %.3g" % (what, rel_l2)


def assert_kept_sets_match(gpu_idx: np.ndarray, ref_idx: np.ndarray, ref_scores: np.ndarray, k: int,
                           band: float = 1e-3):
    """Index sets equal outside a relative band around the k-th largest reference score."""
    for b in range(ref_idx.shape[0]):
        g, r = gpu_idx[b], ref_idx[b]
        assert len(g) == k and len(np.unique(g)) == k, "kept indices must be k distinct values"
        assert np.all(np.diff(g) > 0), "kept indices must be ascending"
        tau = np.sort(ref_scores[b])[::-1][k - 1]
        in_band = np.abs(ref_scores[b] - tau) <= band * abs(tau)
        gs, rs = set(g.tolist()), set(r.tolist())
        diff = gs ^ rs
        bad = [j for j in diff if not in_band[j]]
        assert not bad, "image %d: %d kept indices differ outside the tie band, e.g. %s" % (
            b, len(bad), bad[:5])
