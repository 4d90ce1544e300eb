"""CPU oracle of one pre-LayerNorm transformer block around the sparse attention
(test infrastructure, not product code).

    h = x + Wproj * Attn(LN1(x)) + bproj;   y = h + W2 * gelu(W1 * LN2(h) + b1) + b2

Textbook definitions in float64: LayerNorm over the channel axis with biased variance, exact
(erf) GELU, y = x W^T + b linear maps; the attention and the importance scores are the C
oracle's (paper, Methodology: sparse attention inside the backbone's attention layers, pruning
scores from the global token's attention weights).

Precision.  With storage="f64" (the default, and what the pins check against textbook library
routines) nothing is rounded between the steps except that the C oracle takes q, k, v as float32.
With storage="bf16" every tensor that a bf16 implementation of the block keeps in memory between
two of its steps -- LayerNorm outputs, q/k/v, the attention output, the residual stream after the
projection, the MLP's hidden activations and the block output -- is rounded to bfloat16 (round to
nearest even) at that point, while all arithmetic stays float64.  That is the precision model
"bf16 storage, wide accumulation" of the GPU block; only with it are importance scores of block
and oracle comparable to the 1e-3 tie band, because one bf16 rounding of q or k already moves a
score by about 1e-3 of its value.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf    # the error function as a library routine, float64

from . import cls_scores, ns_attn


def round_bf16(x):
    """float64 -> nearest bfloat16 (ties to even), returned as float64.  Via float32, whose own
    rounding can move a value across a bfloat16 tie in about one case in 2^29."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    odd = (u >> np.uint32(16)) & np.uint32(1)
    r = ((u + np.uint32(0x7FFF) + odd) & np.uint32(0xFFFF0000)).view(np.float32)
    return r.astype(np.float64)


def layer_norm(x, gamma, beta, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gamma + beta


def gelu(x):
    return 0.5 * x * (1.0 + _erf(x / math.sqrt(2.0)))


def patch_embed(pixels, w_patch, b_patch, cls_token, pos_embed, patch):
    """Tokenisation of the ViT backbone, written out from its definition in float64: the pixels
    of patch (pr, pc), in the order (channel, y, x), times the projection matrix, plus bias and the
    patch's position embedding; the CLS token (plus its position embedding) in front.
    pixels [B,ch,gh*patch,gw*patch], w_patch [dim, ch*patch*patch], pos_embed [1+gh*gw, dim]
    -> [B, 1+gh*gw, dim]."""
    px = np.asarray(pixels, dtype=np.float64)
    w = np.asarray(w_patch, dtype=np.float64)
    pos = np.asarray(pos_embed, dtype=np.float64)
    B, ch, hp, wp = px.shape
    gh, gw, dim = hp // patch, wp // patch, w.shape[0]
    out = np.empty((B, 1 + gh * gw, dim), dtype=np.float64)
    out[:, 0, :] = np.asarray(cls_token, dtype=np.float64) + pos[0]
    for b in range(B):
        for pr in range(gh):
            for pc in range(gw):
                v = px[b, :, pr * patch:(pr + 1) * patch, pc * patch:(pc + 1) * patch].reshape(-1)
                n = pr * gw + pc
                out[b, 1 + n, :] = w @ v + np.asarray(b_patch, dtype=np.float64) + pos[1 + n]
    return out


def vit_block(x, w, grid_h, grid_w, block, heads, ln_eps=1e-6, scale=None, coords=None, want_scores=False,
              n_global=1, storage="f64"):
    """x [B,T,dim]; w: dict of numpy arrays named as in the C ABI's ns_vit_block_weights.
    storage: "f64" or "bf16", see the head of this file."""
    assert storage in ("f64", "bf16")
    st = round_bf16 if storage == "bf16" else (lambda t: t)
    x = np.asarray(x, dtype=np.float64)
    B, T, dim = x.shape
    D = dim // heads
    scale = D ** -0.5 if scale is None else scale
    f = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    a = st(layer_norm(x, f["ln1_g"], f["ln1_b"], ln_eps))
    qkv = st(a @ f["w_qkv"].T + f["b_qkv"])                   # [B,T,3*dim], rows q | k | v
    q, k, v = (qkv[..., i * dim:(i + 1) * dim].reshape(B, T, heads, D).transpose(0, 2, 1, 3) for i in range(3))
    att = ns_attn(q, k, v, grid_h, grid_w, block, scale, coords=coords, n_global=n_global)   # [B,H,T,D]
    att = st(att.transpose(0, 2, 1, 3).reshape(B, T, dim))
    h = st(x + att @ f["w_proj"].T + f["b_proj"])
    m = st(gelu(st(layer_norm(h, f["ln2_g"], f["ln2_b"], ln_eps)) @ f["w_fc1"].T + f["b_fc1"]))
    y = st(h + m @ f["w_fc2"].T + f["b_fc2"])
    if want_scores:
        return y, cls_scores(q, k, scale, n_global=n_global)
    return y
