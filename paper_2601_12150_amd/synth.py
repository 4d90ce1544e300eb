"""Seeded synthetic inputs shaped like the paper's high-resolution tiles.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It contains input generation only -- none of the method's
arithmetic (no attention, no scores, no selection) -- and imports neither side.

The paper evaluates on pathology tiles (PANDA, SegPath) run through a trained
backbone; neither is available here, so these generators stand in for them with
the same shapes (patch grids 28^2 ... 256^2 plus one CLS token, 16 heads of 64
channels) and the same structure: smooth spatial correlation and large
"background" regions whose tokens pruning should remove (paper, "Time-Efficiency
Optimization" and the qualitative pruning figure).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    heads: int
    head_dim: int
    grid: int
    block: int
    dtype: str          # "f32" | "bf16"
    keep_pct: int       # percentage of patch tokens kept by the filter
    kind: str           # "iid" | "grf" | "background"
    background: float = 0.0
    seed: int = 0

    @property
    def n_patches(self) -> int:
        return self.grid * self.grid

    @property
    def tokens(self) -> int:
        return 1 + self.n_patches

    @property
    def k(self) -> int:
        # ceil(keep * N) in integer arithmetic
        return (self.n_patches * self.keep_pct + 99) // 100

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


CONFIGS = {
    1: Config("cfg1_g28_b7_f32", 1, 16, 64, 28, 7, "f32", 50, "iid", seed=0),
    2: Config("cfg2_g64_b8_bf16", 4, 16, 64, 64, 8, "bf16", 60, "grf", seed=2),
    3: Config("cfg3_g128_b8_bf16", 2, 16, 64, 128, 8, "bf16", 60, "background", 0.40, seed=3),
    4: Config("cfg4_g256_b16_bf16", 1, 16, 64, 256, 16, "bf16", 40, "background", 0.55, seed=4),
    # Grids the block side does not divide and other window sizes: the paper's 14-pixel patch grids
    # of its 1400- and 3430-pixel inputs (100 and 245 patches per side; "Classification", Table 1),
    # its window-size ablation w in {2, 8, 16, 64} (Tables "window size") on the larger one.
    11: Config("g100_b8_bf16", 2, 16, 64, 100, 8, "bf16", 60, "background", 0.40, seed=11),
    12: Config("g245_b8_bf16", 1, 16, 64, 245, 8, "bf16", 60, "background", 0.40, seed=12),
    13: Config("g245_b16_bf16", 1, 16, 64, 245, 16, "bf16", 60, "background", 0.40, seed=12),
    14: Config("g245_b64_bf16", 1, 16, 64, 245, 64, "bf16", 60, "background", 0.40, seed=12),
    15: Config("g245_b2_bf16", 1, 16, 64, 245, 2, "bf16", 60, "background", 0.40, seed=12),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bfloat16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def _rng(seed: int, stream: int) -> np.random.Generator:
    # counter-based generator: (seed, stream) -> independent reproducible stream
    return np.random.Generator(np.random.Philox(key=[np.uint64(seed), np.uint64(stream)]))


def _finish(x: np.ndarray, dtype: str) -> np.ndarray:
    x = x.astype(np.float32)
    return round_to_bf16(x) if dtype == "bf16" else x


def background_mask(grid: int, fraction: float, seed: int, batch: int,
                    side_lo: int = 8, side_hi: int = 48) -> np.ndarray:
    """[batch, grid, grid] bool: union of seeded axis-aligned rectangles, coverage >= fraction."""
    g = _rng(seed, 1000)
    out = np.zeros((batch, grid, grid), dtype=bool)
    for b in range(batch):
        m = out[b]
        while m.mean() < fraction:
            h = int(g.integers(side_lo, side_hi + 1))
            w = int(g.integers(side_lo, side_hi + 1))
            h, w = min(h, grid), min(w, grid)
            r0 = int(g.integers(0, grid - h + 1))
            c0 = int(g.integers(0, grid - w + 1))
            m[r0:r0 + h, c0:c0 + w] = True
    return out


def _gaussian_field(rng: np.random.Generator, lead_shape, grid: int, sigma: float) -> np.ndarray:
    """Unit-variance smooth random fields on the grid: white noise * Gaussian kernel (wrap)."""
    from scipy.ndimage import gaussian_filter
    w = rng.standard_normal(lead_shape + (grid, grid), dtype=np.float32)
    sig = (0,) * len(lead_shape) + (sigma, sigma)
    f = gaussian_filter(w, sigma=sig, mode="wrap")
    f /= f.std(axis=(-2, -1), keepdims=True)
    return f


def make_qkv(cfg: Config):
    """q, k, v float32 arrays [B,H,T,D] whose values are exactly representable in cfg.dtype.

    Also returns `info` (background mask etc.) for diagnostics."""
    B, H, D, g, T = cfg.batch, cfg.heads, cfg.head_dim, cfg.grid, cfg.tokens
    info = {}
    tensors = []
    bg = None
    if cfg.kind == "background":
        bg = background_mask(g, cfg.background, cfg.seed, B)
        info["background"] = bg
        info["background_fraction"] = float(bg.mean())
    for ti, name in enumerate("qkv"):
        rng = _rng(cfg.seed, ti)
        x = rng.standard_normal((B, H, T, D), dtype=np.float32)
        if cfg.kind == "grf":
            # one smooth field per (tensor, batch, head, channel), length scale 4 patches;
            # the CLS row stays plain N(0,1)
            f = _gaussian_field(_rng(cfg.seed, 10 + ti), (B, H, D), g, 4.0)
            x[:, :, 1:, :] += 0.5 * f.reshape(B, H, D, g * g).transpose(0, 1, 3, 2)
        elif cfg.kind == "background" and name in "kv":
            shared = _rng(cfg.seed, 20 + ti).standard_normal((B, H, 1, D), dtype=np.float32)
            noise = _rng(cfg.seed, 30 + ti).standard_normal((B, H, g * g, D), dtype=np.float32)
            flat = bg.reshape(B, 1, g * g, 1)
            patch = x[:, :, 1:, :]
            x[:, :, 1:, :] = np.where(flat, shared + np.float32(0.01) * noise, patch)
        tensors.append(_finish(x, cfg.dtype))
    return tensors[0], tensors[1], tensors[2], info


def make_tokens(cfg: Config, channels: int = 1024) -> np.ndarray:
    """Token-major activations x [B,T,channels] for the compaction step (values in cfg.dtype)."""
    x = _rng(cfg.seed, 50).standard_normal((cfg.batch, cfg.tokens, channels), dtype=np.float32)
    return _finish(x, cfg.dtype)


def small_case(seed: int, B: int, H: int, D: int, grid_h: int, grid_w: int, dtype: str = "f32",
               n_global: int = 1):
    """iid N(0,1) q, k, v [B,H,G+grid_h*grid_w,D] for unit tests."""
    T = n_global + grid_h * grid_w
    return tuple(_finish(_rng(seed, i).standard_normal((B, H, T, D), dtype=np.float32), dtype)
                 for i in range(3))


def raster_coords(grid_h: int, grid_w: int) -> np.ndarray:
    """Packed (r << 16 | c) of every patch of the full grid, raster order: [grid_h*grid_w] int32."""
    r, c = np.divmod(np.arange(grid_h * grid_w, dtype=np.int64), grid_w)
    return ((r << 16) | c).astype(np.int32)


def make_block_weights(dim: int, mlp_dim: int, seed: int = 0, dtype: str = "bf16", ln_random: bool = False):
    """Random-init weights of one transformer block: matrices ~N(0, 0.02^2) (rounded to `dtype`),
    biases ~N(0, 0.02^2) fp32 (zero-init biases would hide a dropped bias), LayerNorm gamma=1, beta=0
    (or random with ln_random, for tests).  Names as in the C ABI's ns_vit_block_weights."""
    g = _rng(seed, 70)
    def mat(o, i):
        return _finish(np.float32(0.02) * g.standard_normal((o, i), dtype=np.float32), dtype)
    def vec(n):
        return (np.float32(0.02) * g.standard_normal(n, dtype=np.float32)).astype(np.float32)
    w = {"w_qkv": mat(3 * dim, dim), "b_qkv": vec(3 * dim), "w_proj": mat(dim, dim), "b_proj": vec(dim),
         "w_fc1": mat(mlp_dim, dim), "b_fc1": vec(mlp_dim), "w_fc2": mat(dim, mlp_dim), "b_fc2": vec(dim)}
    for n in ("ln1", "ln2"):
        if ln_random:
            w[n + "_g"] = (1.0 + 0.1 * g.standard_normal(dim)).astype(np.float32)
            w[n + "_b"] = (0.1 * g.standard_normal(dim)).astype(np.float32)
        else:
            w[n + "_g"] = np.ones(dim, dtype=np.float32)
            w[n + "_b"] = np.zeros(dim, dtype=np.float32)
    return w


def _fade(t: np.ndarray) -> np.ndarray:
    return t * t * t * (t * (t * 6.0 - 15.0) + 10.0)


def gradient_noise(rng: np.random.Generator, side: int, period: int) -> np.ndarray:
    """[side, side] float32 lattice gradient noise (Perlin's construction): a random unit gradient
    at every lattice point `period` pixels apart; a pixel's value blends the four dot products
    (gradient . offset to the pixel) of its cell's corners with the quintic fade curve.  Values lie
    in about [-0.7, 0.7] and vanish towards the lattice points (pixel centres sit half a pixel off)."""
    n = side // period + 2
    ang = rng.uniform(0.0, 2.0 * np.pi, size=(n, n))
    gy, gx = np.sin(ang).astype(np.float32), np.cos(ang).astype(np.float32)
    p = (np.arange(side, dtype=np.float64) + 0.5) / period
    i = np.floor(p).astype(np.int64)
    f = (p - i).astype(np.float32)
    fy, fx = f[:, None], f[None, :]
    def corner(dy, dx):
        def spread(a):   # lattice values of every pixel's cell corner
            return np.take(np.take(a, i + dy, axis=0), i + dx, axis=1)
        return spread(gy) * (fy - np.float32(dy)) + spread(gx) * (fx - np.float32(dx))
    u, v = _fade(fx), _fade(fy)
    top = corner(0, 0) * (1 - u) + corner(0, 1) * u
    bot = corner(1, 0) * (1 - u) + corner(1, 1) * u
    return (top * (1 - v) + bot * v).astype(np.float32)


def make_tile(seed: int = 5, side: int = 2048, patch: int = 16, background: float = 0.40, batch: int = 1):
    """A synthetic stained-tissue tile: pixels [batch, 3, side, side] float32 (bf16-representable,
    normalised as (p - 0.5) / 0.25 from p in [0, 1]) and the background mask [batch, side/patch,
    side/patch].  Background = the union of seeded rectangles in units of patches (the recipe of
    the 128 x 128 attention workload), near white (0.94 +- 0.02); everywhere else each colour
    channel is a stain-like base colour plus four octaves of seeded gradient noise (periods 256,
    128, 64, 32 pixels, amplitudes halving) and a little pixel noise."""
    g = side // patch
    bg = background_mask(g, background, seed, batch)
    base = np.array([0.72, 0.42, 0.68], dtype=np.float32)
    pixels = np.empty((batch, 3, side, side), dtype=np.float32)
    for b in range(batch):
        mask = np.repeat(np.repeat(bg[b], patch, axis=0), patch, axis=1)
        for c in range(3):
            rng = _rng(seed, 200 + 3 * b + c)
            tissue = np.full((side, side), base[c], dtype=np.float32)
            for o in range(4):
                tissue += np.float32(0.45 / (1 << o)) * gradient_noise(rng, side, 256 >> o)
            tissue += np.float32(0.02) * rng.standard_normal((side, side), dtype=np.float32)
            white = np.float32(0.94) + np.float32(0.02) * rng.uniform(-1.0, 1.0, size=(side, side)).astype(np.float32)
            pixels[b, c] = np.where(mask, white, np.clip(tissue, 0.0, 1.0))
    pixels = (pixels - np.float32(0.5)) / np.float32(0.25)
    return round_to_bf16(pixels), bg


def make_embed_weights(dim: int, patch: int, n_patches: int, channels: int = 3, seed: int = 0, dtype: str = "bf16"):
    """Random-init tokenisation weights: projection [dim, channels*patch*patch], CLS token [dim] and
    position embeddings [1+n_patches, dim] ~N(0, 0.02^2) in `dtype`; projection bias fp32 ~N(0, 0.02^2)."""
    g = _rng(seed, 90)
    def arr(*shape):
        return _finish(np.float32(0.02) * g.standard_normal(shape, dtype=np.float32), dtype)
    return {"w_patch": arr(dim, channels * patch * patch),
            "b_patch": (np.float32(0.02) * g.standard_normal(dim, dtype=np.float32)).astype(np.float32),
            "cls_token": arr(dim), "pos_embed": arr(1 + n_patches, dim)}
