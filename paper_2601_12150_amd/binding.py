"""ctypes binding of libnsattn.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/nsattn.h) and does
nothing but turn torch tensors into device pointers, strides and sizes; all computation runs
in the HIP kernels.  PyTorch supplies device memory and the current stream.  There is no
fallback: if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnsattn.so")

NS_OK, NS_ERR_INVALID_ARG, NS_ERR_UNSUPPORTED, NS_ERR_WORKSPACE, NS_ERR_HIP = range(5)
NS_F32, NS_BF16 = 0, 1

EXPORTS = ["ns_attn_workspace_bytes", "ns_attn_forward", "cls_scores_workspace_bytes", "cls_scores",
           "cls_scores_static_max_bytes", "cls_scores_static",
           "cls_scores_from_logits", "ns_attn_forward_scores", "topk_filter_workspace_bytes", "topk_filter", "topk_filter_global", "vit_forward_features",
           "vit_embed_workspace_bytes", "vit_embed", "vit_block_workspace_bytes", "vit_block_forward", "linear_forward", "vit_workspace_bytes", "vit_forward",
           "vit_stages_workspace_bytes", "vit_forward_stages",
           "ns_attn_patch_kernel_time", "ns_attn_patch_kernel_name", "ns_last_error",
           "ns_version"]


class NsError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("libnsattn error %d: %s" % (code, message))
        self.code = code


class ns_attn_desc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32), ("block", ctypes.c_int32),
                ("radius", ctypes.c_int32), ("n_global", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("tokens", ctypes.c_int32), ("scale", ctypes.c_float),
                ("q_stride_b", ctypes.c_int64), ("q_stride_h", ctypes.c_int64),
                ("q_stride_t", ctypes.c_int64), ("out_stride_b", ctypes.c_int64),
                ("out_stride_h", ctypes.c_int64), ("out_stride_t", ctypes.c_int64),
                ("coords", ctypes.c_void_p)]


class ns_vit_block_desc(ctypes.Structure):
    _fields_ = [("attn", ns_attn_desc), ("dim", ctypes.c_int32), ("mlp_dim", ctypes.c_int32),
                ("ln_eps", ctypes.c_float)]


class ns_vit_block_weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "ln2_g", "ln2_b",
                 "w_fc1", "b_fc1", "w_fc2", "b_fc2")]


class ns_vit_desc(ctypes.Structure):
    _fields_ = [("block", ns_vit_block_desc), ("layers", ctypes.c_int32), ("prune_after", ctypes.c_int32),
                ("keep_k", ctypes.c_int32)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            "%s is missing: build it with `python -m paper_2601_12150_amd.build` "
            "(there is no CPU or PyTorch fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    dp = ctypes.POINTER(ns_attn_desc)
    lib.ns_attn_workspace_bytes.restype = sz
    lib.ns_attn_workspace_bytes.argtypes = [dp]
    lib.ns_attn_forward.restype = ctypes.c_int
    lib.ns_attn_forward.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ns_attn_forward_scores.restype = ctypes.c_int
    lib.ns_attn_forward_scores.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.vit_embed_workspace_bytes.restype = sz
    lib.vit_embed_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, i32]
    lib.vit_embed.restype = ctypes.c_int
    lib.vit_embed.argtypes = [i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.ns_attn_patch_kernel_time.restype = ctypes.c_int
    lib.ns_attn_patch_kernel_time.argtypes = [dp, vp, vp, vp, vp, vp, sz, i32,
                                              ctypes.POINTER(ctypes.c_float), vp]
    lib.cls_scores_workspace_bytes.restype = sz
    lib.ns_attn_patch_kernel_name.restype = ctypes.c_char_p
    lib.ns_attn_patch_kernel_name.argtypes = [dp]
    lib.cls_scores_workspace_bytes.argtypes = [dp]
    lib.cls_scores.restype = ctypes.c_int
    lib.cls_scores.argtypes = [dp, vp, vp, vp, vp, sz, vp]
    lib.cls_scores_static_max_bytes.restype = sz
    lib.cls_scores_static_max_bytes.argtypes = []
    lib.cls_scores_static.restype = ctypes.c_int
    lib.cls_scores_static.argtypes = [dp, vp, vp, vp, vp]
    lib.cls_scores_from_logits.restype = ctypes.c_int
    lib.cls_scores_from_logits.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp]
    lib.topk_filter_workspace_bytes.restype = sz
    lib.topk_filter_workspace_bytes.argtypes = [i32, i32, i32]
    lib.topk_filter.restype = ctypes.c_int
    lib.topk_filter.argtypes = [i32, i32, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.topk_filter_global.restype = ctypes.c_int
    lib.topk_filter_global.argtypes = [i32, i32, i32, i32, vp, vp, i32, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.vit_block_workspace_bytes.restype = sz
    lib.vit_block_workspace_bytes.argtypes = [ctypes.POINTER(ns_vit_block_desc)]
    lib.vit_block_forward.restype = ctypes.c_int
    lib.vit_block_forward.argtypes = [ctypes.POINTER(ns_vit_block_desc),
                                      ctypes.POINTER(ns_vit_block_weights), vp, vp, vp, vp, sz, vp]
    lib.vit_workspace_bytes.restype = sz
    lib.vit_workspace_bytes.argtypes = [ctypes.POINTER(ns_vit_desc)]
    lib.linear_forward.restype = ctypes.c_int
    lib.linear_forward.argtypes = [i32, i32, i32, vp, vp, vp, vp, i32, vp, vp]
    lib.vit_forward.restype = ctypes.c_int
    lib.vit_forward.argtypes = [ctypes.POINTER(ns_vit_desc), ctypes.POINTER(ns_vit_block_weights), vp, vp, vp, vp,
                                sz, vp]
    lib.vit_forward_features.restype = ctypes.c_int
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.vit_stages_workspace_bytes.restype = ctypes.c_size_t
    lib.vit_stages_workspace_bytes.argtypes = [ctypes.POINTER(ns_vit_desc), ctypes.c_int32, i32p, i32p]
    lib.vit_forward_stages.restype = ctypes.c_int
    lib.vit_forward_stages.argtypes = [ctypes.POINTER(ns_vit_desc), ctypes.c_int32, i32p, i32p,
                                       ctypes.POINTER(ns_vit_block_weights), vp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.vit_forward_features.argtypes = [ctypes.POINTER(ns_vit_desc), ctypes.POINTER(ns_vit_block_weights), vp, vp,
                                         vp, i32, ctypes.POINTER(i32), ctypes.POINTER(vp), vp, sz, vp]
    lib.ns_last_error.restype = ctypes.c_char_p
    lib.ns_version.restype = ctypes.c_char_p
    return lib


lib = _load()


def _check(code: int) -> None:
    if code != NS_OK:
        raise NsError(code, lib.ns_last_error().decode())


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return NS_F32
    if t.dtype == torch.bfloat16:
        return NS_BF16
    raise TypeError("only float32 and bfloat16 tensors are supported, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> Optional[torch.Tensor]:
    if nbytes == 0:
        return workspace
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return workspace


def make_desc(q: torch.Tensor, grid_h: int, grid_w: int, block: int, scale: Optional[float] = None,
              out: Optional[torch.Tensor] = None, coords: Optional[torch.Tensor] = None,
              radius: int = 1, n_global: int = 1) -> ns_attn_desc:
    """Descriptor for q (and k, v with the same strides) of shape [B,H,T,D]."""
    B, H, T, D = q.shape
    if q.stride(3) != 1:
        raise ValueError("head_dim must be contiguous")
    d = ns_attn_desc()
    d.batch, d.heads, d.head_dim = B, H, D
    d.grid_h, d.grid_w, d.block, d.radius, d.n_global = grid_h, grid_w, block, radius, n_global
    d.dtype = _dtype_code(q)
    d.tokens = T
    d.scale = float(D) ** -0.5 if scale is None else float(scale)
    d.q_stride_b, d.q_stride_h, d.q_stride_t = q.stride(0), q.stride(1), q.stride(2)
    if out is not None:
        d.out_stride_b, d.out_stride_h, d.out_stride_t = out.stride(0), out.stride(1), out.stride(2)
    d.coords = None if coords is None else coords.data_ptr()
    return d


def ns_attn_forward(q, k, v, grid_h, grid_w, block, scale=None, coords=None, out=None,
                    want_cls=False, workspace=None, stream=None, radius=1, n_global=1):
    """Neighbourhood-sparse attention.  q, k, v: [B,H,T,D] device tensors with equal strides.

    Returns out [B,H,T,D] (allocated contiguous unless given) and, with want_cls, also the
    global query's logits [B,H,T] and log-sum-exp [B,H] (both fp32; [B,H,G,T] and [B,H,G] when
    n_global = G > 1)."""
    if not (q.shape == k.shape == v.shape and q.stride() == k.stride() == v.stride()):
        raise ValueError("q, k, v must have the same shape and strides")
    if not (q.dtype == k.dtype == v.dtype):
        raise ValueError("q, k, v must have the same dtype")
    B, H, T, D = q.shape
    if out is None:
        out = torch.empty((B, H, T, D), dtype=q.dtype, device=q.device)
    if coords is not None and (coords.dtype != torch.int32 or not coords.is_contiguous()):
        raise ValueError("coords must be a contiguous int32 tensor [B, T - n_global]")
    desc = make_desc(q, grid_h, grid_w, block, scale, out, coords, radius, n_global)
    logits = lse = None
    if want_cls:
        G = int(n_global)
        logits = torch.empty((B, H, T) if G == 1 else (B, H, G, T), dtype=torch.float32, device=q.device)
        lse = torch.empty((B, H) if G == 1 else (B, H, G), dtype=torch.float32, device=q.device)
    nbytes = lib.ns_attn_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, q.device, workspace)
    _check(lib.ns_attn_forward(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(logits),
                               _ptr(lse), _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream)))
    return (out, logits, lse) if want_cls else out


def ns_attn_forward_scores(q, k, v, grid_h, grid_w, block, scale=None, coords=None, out=None,
                           workspace=None, stream=None, n_global=1):
    """ns_attn_forward with the global queries' by-products, and the importance scores of the
    patches from them, in one call.  Returns (out, cls_logits, cls_lse, scores [B, T - n_global])."""
    if not (q.shape == k.shape == v.shape and q.stride() == k.stride() == v.stride()):
        raise ValueError("q, k, v must have the same shape and strides")
    if not (q.dtype == k.dtype == v.dtype):
        raise ValueError("q, k, v must have the same dtype")
    B, H, T, D = q.shape
    G = int(n_global)
    if out is None:
        out = torch.empty((B, H, T, D), dtype=q.dtype, device=q.device)
    if coords is not None and (coords.dtype != torch.int32 or not coords.is_contiguous()):
        raise ValueError("coords must be a contiguous int32 tensor [B, T - n_global]")
    desc = make_desc(q, grid_h, grid_w, block, scale, out, coords, 1, n_global)
    logits = torch.empty((B, H, T) if G == 1 else (B, H, G, T), dtype=torch.float32, device=q.device)
    lse = torch.empty((B, H) if G == 1 else (B, H, G), dtype=torch.float32, device=q.device)
    scores = torch.empty((B, T - G), dtype=torch.float32, device=q.device)
    nbytes = lib.ns_attn_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, q.device, workspace)
    _check(lib.ns_attn_forward_scores(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(logits),
                                      _ptr(lse), _ptr(scores), _ptr(ws), 0 if ws is None else ws.numel(),
                                      _stream(stream)))
    return out, logits, lse, scores


def ns_attn_patch_kernel_time(q, k, v, grid_h, grid_w, block, scale=None, coords=None, out=None,
                              reps=10, workspace=None, stream=None) -> float:
    """Average duration in ms of one launch of the patch-query attention kernel (HIP events
    on the launch stream; this call waits for the GPU)."""
    B, H, T, D = q.shape
    if out is None:
        out = torch.empty((B, H, T, D), dtype=q.dtype, device=q.device)
    desc = make_desc(q, grid_h, grid_w, block, scale, out, coords)
    nbytes = lib.ns_attn_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, q.device, workspace)
    ms = ctypes.c_float(0.0)
    _check(lib.ns_attn_patch_kernel_time(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(ws),
                                         0 if ws is None else ws.numel(), int(reps), ctypes.byref(ms),
                                         _stream(stream)))
    return float(ms.value)


def ns_attn_patch_kernel_name(q, grid_h, grid_w, block, scale=None, coords=None, n_global=1) -> str:
    """Name of the kernel ns_attn_forward launches for the patch queries of this problem."""
    B, H, T, D = q.shape
    desc = make_desc(q, grid_h, grid_w, block, scale, None, coords, 1, n_global)
    desc.out_stride_b, desc.out_stride_h, desc.out_stride_t = desc.q_stride_b, desc.q_stride_h, desc.q_stride_t
    return lib.ns_attn_patch_kernel_name(ctypes.byref(desc)).decode()


def cls_scores(q, k, scale=None, n_global=1, scores=None, workspace=None, stream=None):
    """Head-averaged softmax weight of the global query on every patch key: [B, T-G] fp32."""
    if not (q.shape == k.shape and q.stride() == k.stride() and q.dtype == k.dtype):
        raise ValueError("q and k must have the same shape, strides and dtype")
    B, H, T, D = q.shape
    # the grid fields are not used by scoring; a 1 x (T-G) grid keeps the descriptor valid
    desc = make_desc(q, 1, T - n_global, 1, scale, None, None, 1, n_global)
    if scores is None:
        scores = torch.empty((B, T - n_global), dtype=torch.float32, device=q.device)
    nbytes = lib.cls_scores_workspace_bytes(ctypes.byref(desc))
    ws = _workspace(nbytes, q.device, workspace)
    _check(lib.cls_scores(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(scores), _ptr(ws),
                          0 if ws is None else ws.numel(), _stream(stream)))
    return scores


def cls_scores_static(q, k, scale=None, n_global=1, scores=None, stream=None):
    """cls_scores on the library's own scratch buffer: the call allocates nothing when `scores` is given."""
    if not (q.shape == k.shape and q.stride() == k.stride() and q.dtype == k.dtype):
        raise ValueError("q and k must have the same shape, strides and dtype")
    B, H, T, D = q.shape
    desc = make_desc(q, 1, T - n_global, 1, scale, None, None, 1, n_global)
    if scores is None:
        scores = torch.empty((B, T - n_global), dtype=torch.float32, device=q.device)
    _check(lib.cls_scores_static(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(scores), _stream(stream)))
    return scores


def cls_scores_from_logits(cls_logits, cls_lse, n_global=1, scores=None, stream=None):
    """The same scores from ns_attn_forward's by-products (no second pass over K)."""
    B, H, T = cls_logits.shape[0], cls_logits.shape[1], cls_logits.shape[-1]
    if cls_logits.dim() == 4 and cls_logits.shape[2] != n_global:
        raise ValueError("cls_logits must be [B,H,G,T] with G = n_global")
    if not (cls_logits.is_contiguous() and cls_lse.is_contiguous()):
        raise ValueError("cls_logits and cls_lse must be contiguous")
    if scores is None:
        scores = torch.empty((B, T - n_global), dtype=torch.float32, device=cls_logits.device)
    _check(lib.cls_scores_from_logits(B, H, T, n_global, _ptr(cls_logits), _ptr(cls_lse),
                                      _ptr(scores), _stream(stream)))
    return scores


def topk_filter(scores, k, x=None, coords=None, kept_idx=None, y=None, coords_out=None,
                workspace=None, stream=None, n_global=1):
    """Keep the k best-scoring patches per image.

    scores [B,N] fp32; x optional [B,G+N,C] (G = n_global leading rows are kept); coords optional
    [B,N] int32.
    Returns (kept_idx [B,k] int32 ascending, y [B,G+k,C] or None, coords_out [B,k] or None)."""
    G = int(n_global)
    if scores.dtype != torch.float32 or not scores.is_contiguous():
        raise ValueError("scores must be a contiguous float32 tensor")
    B, N = scores.shape
    dev = scores.device
    kk = max(int(k), 0)
    if kept_idx is None:
        kept_idx = torch.empty((B, kk), dtype=torch.int32, device=dev)
    C, xdt = 0, NS_BF16
    if x is not None:
        if not x.is_contiguous() or x.shape[0] != B or x.shape[1] != G + N:
            raise ValueError("x must be contiguous [B, n_global+N, C]")
        C, xdt = x.shape[2], _dtype_code(x)
        if y is None:
            y = torch.empty((B, G + kk, C), dtype=x.dtype, device=dev)
    if coords is not None:
        if coords.dtype != torch.int32 or not coords.is_contiguous():
            raise ValueError("coords must be contiguous int32 [B,N]")
        if coords_out is None:
            coords_out = torch.empty((B, kk), dtype=torch.int32, device=dev)
    nbytes = lib.topk_filter_workspace_bytes(B, N, int(k))
    ws = _workspace(nbytes, dev, workspace)
    if G == 1:
        _check(lib.topk_filter(B, N, int(k), _ptr(scores), _ptr(x), C, xdt, _ptr(coords), _ptr(kept_idx),
                               _ptr(y), _ptr(coords_out), _ptr(ws), 0 if ws is None else ws.numel(),
                               _stream(stream)))
    else:
        _check(lib.topk_filter_global(B, N, int(k), G, _ptr(scores), _ptr(x), C, xdt, _ptr(coords),
                                      _ptr(kept_idx), _ptr(y), _ptr(coords_out), _ptr(ws),
                                      0 if ws is None else ws.numel(), _stream(stream)))
    return kept_idx, y, coords_out


def vit_embed(pixels, w_patch, b_patch, cls_token, pos_embed, patch, out=None, workspace=None, stream=None):
    """Patch embedding: pixels [B,channels,gh*patch,gw*patch] bf16 -> tokens [B, 1+gh*gw, dim] bf16
    (CLS token in front, position embeddings added).  w_patch [dim, channels*patch*patch] bf16,
    b_patch [dim] fp32, cls_token [dim] bf16, pos_embed [1+gh*gw, dim] bf16."""
    for name, t, dt in (("pixels", pixels, torch.bfloat16), ("w_patch", w_patch, torch.bfloat16),
                        ("b_patch", b_patch, torch.float32), ("cls_token", cls_token, torch.bfloat16),
                        ("pos_embed", pos_embed, torch.bfloat16)):
        if t.dtype != dt or not t.is_contiguous():
            raise ValueError("%s must be a contiguous %s tensor" % (name, dt))
    B, ch, hp, wp = pixels.shape
    if hp % patch or wp % patch:
        raise ValueError("image sides must be multiples of the patch side")
    gh, gw, dim = hp // patch, wp // patch, w_patch.shape[0]
    if w_patch.shape[1] != ch * patch * patch or pos_embed.shape != (1 + gh * gw, dim):
        raise ValueError("w_patch must be [dim, channels*patch*patch] and pos_embed [1+gh*gw, dim]")
    if out is None:
        out = torch.empty((B, 1 + gh * gw, dim), dtype=torch.bfloat16, device=pixels.device)
    nbytes = lib.vit_embed_workspace_bytes(B, ch, gh, gw, patch, dim)
    ws = _workspace(max(nbytes, 1), pixels.device, workspace)
    _check(lib.vit_embed(B, ch, gh, gw, patch, dim, _ptr(pixels), _ptr(w_patch), _ptr(b_patch), _ptr(cls_token),
                         _ptr(pos_embed), _ptr(out), _ptr(ws), ws.numel(), _stream(stream)))
    return out


WEIGHT_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj", "ln2_g", "ln2_b",
                "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def vit_block_forward(x, weights, grid_h, grid_w, block, heads, ln_eps=1e-6, scale=None, coords=None,
                      want_scores=False, out=None, workspace=None, stream=None, n_global=1):
    """One pre-LayerNorm transformer block around the sparse attention.

    x [B,T,dim] bf16 contiguous; weights: dict of device tensors (matrices bf16 [out,in], vectors
    fp32).  Returns x_out [B,T,dim] (and the importance scores [B,T-n_global] with want_scores)."""
    if x.dtype != torch.bfloat16 or not x.is_contiguous():
        raise ValueError("x must be a contiguous bfloat16 tensor [B,T,dim]")
    B, T, dim = x.shape
    for n in WEIGHT_NAMES:
        t = weights[n]
        want = torch.bfloat16 if n.startswith("w_") else torch.float32
        if t.dtype != want or not t.is_contiguous() or t.device != x.device:
            raise ValueError("weight %s must be a contiguous %s tensor on %s" % (n, want, x.device))
    mlp = weights["w_fc1"].shape[0]
    d = ns_vit_block_desc()
    a = d.attn
    a.batch, a.heads, a.head_dim = B, heads, dim // heads
    a.grid_h, a.grid_w, a.block, a.radius, a.n_global = grid_h, grid_w, block, 1, int(n_global)
    a.dtype, a.tokens = NS_BF16, T
    a.scale = float(dim // heads) ** -0.5 if scale is None else float(scale)
    if coords is not None:
        if coords.dtype != torch.int32 or not coords.is_contiguous():
            raise ValueError("coords must be a contiguous int32 tensor [B, T-1]")
        a.coords = coords.data_ptr()
    d.dim, d.mlp_dim, d.ln_eps = dim, mlp, float(ln_eps)
    w = ns_vit_block_weights()
    for n in WEIGHT_NAMES:
        setattr(w, n, weights[n].data_ptr())
    if out is None:
        out = torch.empty_like(x)
    scores = torch.empty((B, T - int(n_global)), dtype=torch.float32, device=x.device) if want_scores else None
    nbytes = lib.vit_block_workspace_bytes(ctypes.byref(d))
    ws = _workspace(max(nbytes, 1), x.device, workspace)
    _check(lib.vit_block_forward(ctypes.byref(d), ctypes.byref(w), _ptr(x), _ptr(out), _ptr(scores), _ptr(ws),
                                 ws.numel(), _stream(stream)))
    return (out, scores) if want_scores else out


def linear_forward(x, w, bias, residual=None, gelu=False, out=None, stream=None):
    """y = act(x w^T + bias) + residual; x [M,K] bf16, w [N,K] bf16, bias [N] fp32, residual [M,N] bf16."""
    for t, dt in ((x, torch.bfloat16), (w, torch.bfloat16), (bias, torch.float32)):
        if t.dtype != dt or not t.is_contiguous():
            raise ValueError("x, w must be contiguous bfloat16 and bias contiguous float32")
    M, K = x.shape
    N = w.shape[0]
    if w.shape[1] != K or bias.numel() != N:
        raise ValueError("shape mismatch")
    if residual is not None and (residual.dtype != torch.bfloat16 or not residual.is_contiguous()
                                 or tuple(residual.shape) != (M, N)):
        raise ValueError("residual must be a contiguous bfloat16 tensor [M,N]")
    if out is None:
        out = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _check(lib.linear_forward(M, N, K, _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), 1 if gelu else 0, _ptr(out),
                              _stream(stream)))
    return out


def vit_forward(x, layer_weights, grid_h, grid_w, block, heads, prune_after=0, keep_k=0, ln_eps=1e-6,
                scale=None, out=None, workspace=None, stream=None, n_global=1, tap_layers=None):
    """A stack of blocks with one pruning stage after block `prune_after` (keep_k patches kept).

    x [B,T,dim] bf16; layer_weights: list of weight dicts (see vit_block_forward).
    Returns (x_out [B, n_global+keep_k or T, dim], kept_idx [B,keep_k] or None); with tap_layers
    (ascending 1-based block numbers) also a list of feature maps [B, grid_h*grid_w, dim], the patch
    tokens after those blocks in raster order."""
    if x.dtype != torch.bfloat16 or not x.is_contiguous():
        raise ValueError("x must be a contiguous bfloat16 tensor [B,T,dim]")
    B, T, dim = x.shape
    d = ns_vit_desc()
    a = d.block.attn
    a.batch, a.heads, a.head_dim = B, heads, dim // heads
    a.grid_h, a.grid_w, a.block, a.radius, a.n_global = grid_h, grid_w, block, 1, int(n_global)
    a.dtype, a.tokens = NS_BF16, T
    a.scale = float(dim // heads) ** -0.5 if scale is None else float(scale)
    d.block.dim, d.block.mlp_dim, d.block.ln_eps = dim, layer_weights[0]["w_fc1"].shape[0], float(ln_eps)
    d.layers, d.prune_after, d.keep_k = len(layer_weights), int(prune_after), int(keep_k)
    warr = (ns_vit_block_weights * len(layer_weights))()
    for i, lw in enumerate(layer_weights):
        for n in WEIGHT_NAMES:
            t = lw[n]
            want = torch.bfloat16 if n.startswith("w_") else torch.float32
            if t.dtype != want or not t.is_contiguous() or t.device != x.device:
                raise ValueError("layer %d weight %s must be a contiguous %s tensor on %s" % (i, n, want, x.device))
            setattr(warr[i], n, t.data_ptr())
    pruning = prune_after > 0 and keep_k > 0
    if out is None:
        out = torch.empty((B, int(n_global) + keep_k if pruning else T, dim), dtype=x.dtype, device=x.device)
    kept = torch.empty((B, keep_k), dtype=torch.int32, device=x.device) if pruning else None
    nbytes = lib.vit_workspace_bytes(ctypes.byref(d))
    ws = _workspace(max(nbytes, 1), x.device, workspace)
    if tap_layers is None:
        _check(lib.vit_forward(ctypes.byref(d), warr, _ptr(x), _ptr(out), _ptr(kept), _ptr(ws), ws.numel(),
                               _stream(stream)))
        return out, kept
    taps = [torch.empty((B, grid_h * grid_w, dim), dtype=x.dtype, device=x.device) for _ in tap_layers]
    tl = (ctypes.c_int32 * len(taps))(*[int(t) for t in tap_layers])
    tp = (ctypes.c_void_p * len(taps))(*[t.data_ptr() for t in taps])
    _check(lib.vit_forward_features(ctypes.byref(d), warr, _ptr(x), _ptr(out), _ptr(kept), len(taps), tl, tp,
                                    _ptr(ws), ws.numel(), _stream(stream)))
    return out, kept, taps


def vit_forward_stages(x, layer_weights, grid_h, grid_w, block, heads, stage_after, stage_keep, ln_eps=1e-6,
                       scale=None, out=None, workspace=None, stream=None, n_global=1):
    """The stack with several pruning stages: after block stage_after[i] (1-based, ascending) the
    stage_keep[i] best-scoring of the patches still present are kept.

    Returns (x_out [B, n_global + stage_keep[-1], dim], kept_idx [B, stage_keep[-1]] original patch
    indices, ascending); without stages (x_out [B,T,dim], None)."""
    if x.dtype != torch.bfloat16 or not x.is_contiguous():
        raise ValueError("x must be a contiguous bfloat16 tensor [B,T,dim]")
    B, T, dim = x.shape
    d = ns_vit_desc()
    a = d.block.attn
    a.batch, a.heads, a.head_dim = B, heads, dim // heads
    a.grid_h, a.grid_w, a.block, a.radius, a.n_global = grid_h, grid_w, block, 1, int(n_global)
    a.dtype, a.tokens = NS_BF16, T
    a.scale = float(dim // heads) ** -0.5 if scale is None else float(scale)
    d.block.dim, d.block.mlp_dim, d.block.ln_eps = dim, layer_weights[0]["w_fc1"].shape[0], float(ln_eps)
    d.layers = len(layer_weights)
    warr = (ns_vit_block_weights * len(layer_weights))()
    for i, lw in enumerate(layer_weights):
        for n in WEIGHT_NAMES:
            t = lw[n]
            want = torch.bfloat16 if n.startswith("w_") else torch.float32
            if t.dtype != want or not t.is_contiguous() or t.device != x.device:
                raise ValueError("layer %d weight %s must be a contiguous %s tensor on %s" % (i, n, want, x.device))
            setattr(warr[i], n, t.data_ptr())
    ns = len(stage_after)
    if len(stage_keep) != ns:
        raise ValueError("stage_after and stage_keep must have the same length")
    aft = (ctypes.c_int32 * max(ns, 1))(*[int(v) for v in stage_after])
    kp = (ctypes.c_int32 * max(ns, 1))(*[int(v) for v in stage_keep])
    k_last = int(stage_keep[-1]) if ns else 0
    if out is None:
        out = torch.empty((B, int(n_global) + k_last if ns else T, dim), dtype=x.dtype, device=x.device)
    kept = torch.empty((B, k_last), dtype=torch.int32, device=x.device) if ns else None
    nbytes = lib.vit_stages_workspace_bytes(ctypes.byref(d), ns, aft, kp)
    ws = _workspace(max(nbytes, 1), x.device, workspace)
    _check(lib.vit_forward_stages(ctypes.byref(d), ns, aft, kp, warr, _ptr(x), _ptr(out), _ptr(kept), _ptr(ws),
                                  ws.numel(), _stream(stream)))
    return out, kept
