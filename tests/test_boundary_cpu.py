"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every function
the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nsattn.h")


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{]*\)\s*;", text)
    return sorted(set(names))


def test_library_exports_every_declared_function(nb):
    names = declared_functions()
    assert {"ns_attn_forward", "cls_scores", "topk_filter", "vit_block_forward"} <= set(names)
    raw = ctypes.CDLL(nb.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), "libnsattn.so does not export %s" % n
    assert set(nb.EXPORTS) == set(names)


def good_desc(nb):
    d = nb.ns_attn_desc()
    d.batch, d.heads, d.head_dim = 1, 2, 64
    d.grid_h = d.grid_w = 8
    d.block, d.radius, d.n_global, d.dtype, d.tokens = 4, 1, 1, nb.NS_BF16, 65
    d.scale = 0.125
    d.q_stride_b, d.q_stride_h, d.q_stride_t = 2 * 65 * 64, 65 * 64, 64
    d.out_stride_b, d.out_stride_h, d.out_stride_t = 2 * 65 * 64, 65 * 64, 64
    return d


FAKE = ctypes.c_void_p(0x10000)   # never dereferenced: every call below fails validation first


def attn_call(nb, d, q=FAKE, out=ctypes.c_void_p(0x20000), ws=ctypes.c_void_p(0x30000), ws_bytes=1 << 30):
    return nb.lib.ns_attn_forward(ctypes.byref(d), q, FAKE, FAKE, out, None, None, ws, ws_bytes, None)


def test_descriptor_validation(nb):
    d = good_desc(nb)
    assert nb.lib.ns_attn_workspace_bytes(ctypes.byref(d)) > 0
    cases = [("batch", 0, nb.NS_ERR_INVALID_ARG), ("heads", -1, nb.NS_ERR_INVALID_ARG),
             ("block", 0, nb.NS_ERR_INVALID_ARG), ("dtype", 7, nb.NS_ERR_INVALID_ARG),
             ("tokens", 64, nb.NS_ERR_INVALID_ARG), ("scale", float("nan"), nb.NS_ERR_INVALID_ARG),
             ("q_stride_t", 63, nb.NS_ERR_INVALID_ARG), ("q_stride_h", 65 * 64 + 1, nb.NS_ERR_INVALID_ARG),
             ("out_stride_t", 8, nb.NS_ERR_INVALID_ARG),
             ("head_dim", 128, nb.NS_ERR_UNSUPPORTED), ("radius", 2, nb.NS_ERR_UNSUPPORTED),
             ("n_global", 300, nb.NS_ERR_UNSUPPORTED), ("n_global", 0, nb.NS_ERR_INVALID_ARG)]
    for field, value, code in cases:
        d = good_desc(nb)
        setattr(d, field, value)
        if field == "n_global":
            d.tokens = 64 + value
        assert attn_call(nb, d) == code, field
        assert nb.lib.ns_last_error()
        assert nb.lib.ns_attn_workspace_bytes(ctypes.byref(d)) == 0
    assert nb.lib.ns_attn_forward(None, FAKE, FAKE, FAKE, FAKE, None, None, None, 0, None) == nb.NS_ERR_INVALID_ARG


def test_pointer_and_workspace_validation(nb):
    d = good_desc(nb)
    assert attn_call(nb, d, q=None) == nb.NS_ERR_INVALID_ARG
    assert attn_call(nb, d, q=ctypes.c_void_p(0x10008)) == nb.NS_ERR_INVALID_ARG       # misaligned
    assert attn_call(nb, d, out=FAKE) == nb.NS_ERR_INVALID_ARG                         # aliasing
    assert attn_call(nb, d, ws=None) == nb.NS_ERR_WORKSPACE
    assert attn_call(nb, d, ws=ctypes.c_void_p(0x30010)) == nb.NS_ERR_WORKSPACE        # misaligned
    assert attn_call(nb, d, ws_bytes=16) == nb.NS_ERR_WORKSPACE
    assert b"needed" in nb.lib.ns_last_error()


def test_forward_scores_validation(nb):
    L, d = nb.lib, good_desc(nb)
    out, ws = ctypes.c_void_p(0x20000), ctypes.c_void_p(0x30000)
    def call(logits=FAKE, scores=FAKE, desc=d):
        return L.ns_attn_forward_scores(ctypes.byref(desc), FAKE, FAKE, FAKE, out, logits, None, scores, ws, 1 << 30, None)
    assert call(logits=None) == nb.NS_ERR_INVALID_ARG            # the scoring reads the logits back
    assert call(scores=None) == nb.NS_ERR_INVALID_ARG
    assert call(scores=ctypes.c_void_p(0x10002)) == nb.NS_ERR_INVALID_ARG
    bad = good_desc(nb)
    bad.heads = 0
    assert call(desc=bad) == nb.NS_ERR_INVALID_ARG


def test_topk_and_scores_validation(nb):
    L = nb.lib
    args = dict(x=None, C=0, dt=nb.NS_BF16, cin=None, kept=FAKE, y=None, cout=None)
    def call(B, N, k, scores=FAKE, **kw):
        a = dict(args); a.update(kw)
        return L.topk_filter(B, N, k, scores, a["x"], a["C"], a["dt"], a["cin"], a["kept"], a["y"],
                             a["cout"], None, 0, None)
    assert call(1, 100, 0) == nb.NS_ERR_INVALID_ARG
    assert call(1, 100, 101) == nb.NS_ERR_INVALID_ARG
    assert call(0, 100, 10) == nb.NS_ERR_INVALID_ARG
    assert call(1, 100, 10, scores=None) == nb.NS_ERR_INVALID_ARG
    assert call(1, 100, 10, x=FAKE, C=64) == nb.NS_ERR_INVALID_ARG                   # y missing
    assert call(1, 100, 10, x=FAKE, y=ctypes.c_void_p(0x20000), C=3) == nb.NS_ERR_UNSUPPORTED
    assert call(1, 100, 10, cin=FAKE) == nb.NS_ERR_INVALID_ARG                       # coords_out missing
    # rows above 32768 scores need a workspace (several workgroups per image)
    assert L.topk_filter_workspace_bytes(4, 16384, 100) == 0
    assert L.topk_filter_workspace_bytes(1, 32768, 100) == 0
    assert L.topk_filter_workspace_bytes(1, 70001, 100) == 4 * 69 * 1024 + 4 * 8 + 69 * 4
    assert L.topk_filter_workspace_bytes(2, 300000, 100) == 2 * (4 * 98 * 1024 + 4 * 8 + 98 * 4)   # 3 keys per thread
    assert call(1, 70001, 10) == nb.NS_ERR_WORKSPACE
    assert b"needed" in nb.lib.ns_last_error()
    assert L.cls_scores_from_logits(1, 2, 1, 1, FAKE, FAKE, FAKE, None) == nb.NS_ERR_INVALID_ARG
    assert L.cls_scores_from_logits(1, 2, 10, 1, None, FAKE, FAKE, None) == nb.NS_ERR_INVALID_ARG
    d = good_desc(nb)
    assert L.cls_scores(ctypes.byref(d), FAKE, FAKE, None, FAKE, 1 << 30, None) == nb.NS_ERR_INVALID_ARG
    assert L.cls_scores_workspace_bytes(ctypes.byref(d)) > 0


def test_embed_validation(nb):
    L = nb.lib
    assert L.vit_embed_workspace_bytes(1, 3, 128, 128, 14, 1024) == 16384 * 640 * 2 + 1024 * 640 * 2   # 588 -> 640 columns
    assert L.vit_embed_workspace_bytes(1, 3, 8, 8, 16, 100) == 0                                      # dim % 128
    def call(B=1, ch=3, gh=8, gw=8, ps=14, dim=512, px=FAKE, w=FAKE, ws=FAKE, ws_bytes=1 << 30):
        return L.vit_embed(B, ch, gh, gw, ps, dim, px, w, FAKE, FAKE, FAKE, FAKE, ws, ws_bytes, None)
    assert call(B=0) == nb.NS_ERR_INVALID_ARG
    assert call(dim=100) == nb.NS_ERR_UNSUPPORTED
    assert call(px=None) == nb.NS_ERR_INVALID_ARG
    assert call(w=ctypes.c_void_p(0x10008)) == nb.NS_ERR_INVALID_ARG          # misaligned
    assert call(ws=None) == nb.NS_ERR_WORKSPACE
    assert call(ws_bytes=1024) == nb.NS_ERR_WORKSPACE


def test_kernel_choice_policy(nb, monkeypatch):
    """Which kernel serves which problem (host logic; without a device the CU count defaults to 256)."""
    monkeypatch.delenv("NSATTN_KERNEL", raising=False)

    def desc(B, H, g, block, dtype=None, coords=False):
        d = nb.ns_attn_desc()
        d.batch, d.heads, d.head_dim = B, H, 64
        d.grid_h = d.grid_w = g
        d.block, d.radius, d.n_global = block, 1, 1
        d.dtype = nb.NS_BF16 if dtype is None else dtype
        d.tokens = 1 + g * g if not coords else 1 + (g * g) // 2
        d.scale = 0.125
        T = d.tokens
        d.q_stride_b, d.q_stride_h, d.q_stride_t = H * T * 64, T * 64, 64
        d.out_stride_b, d.out_stride_h, d.out_stride_t = H * T * 64, T * 64, 64
        d.coords = 0x40000 if coords else None
        return d

    name = lambda d: nb.lib.ns_attn_patch_kernel_name(ctypes.byref(d)).decode()
    assert name(desc(2, 16, 128, 8)) == "attn_sweep_kernel"            # 512 rows of blocks
    assert name(desc(1, 4, 24, 8)) == "attn_mfma_persist_kernel"        # too few rows of blocks for the sweep
    assert name(desc(1, 16, 256, 16)) == "attn_block16_kernel"          # 16x16 blocks, 4096 of them
    assert name(desc(1, 2, 32, 16)) == "attn_mfma_persist_kernel"       # 16x16 blocks, too few for a workgroup each
    assert name(desc(1, 2, 8, 8)) == "attn_mfma_kernel"                 # a single block
    assert name(desc(1, 2, 24, 8, dtype=nb.NS_F32)) == "attn_generic_kernel"
    assert name(desc(1, 2, 24, 4)) == "attn_mfma_ragged_kernel"         # 4x4 blocks on the full grid
    assert name(desc(1, 16, 100, 8)) == "attn_mfma_ragged_kernel"       # the block side does not divide the grid
    assert name(desc(2, 16, 100, 8)) == "attn_sweep_kernel"             # ... 416 rows of blocks: short edge blocks in the sweep
    assert name(desc(1, 16, 245, 2)) == "attn_sweep_kernel"             # 2x2 blocks on the sweep's 8x8 tiles (496 rows of tiles)
    assert name(desc(1, 16, 245, 3)) == "attn_mfma_ragged_kernel"       # 3 does not divide 8
    assert name(desc(1, 16, 245, 16)) == "attn_block16_kernel"          # short edge blocks in the 16x16 kernel
    assert name(desc(1, 16, 245, 64)) == "attn_block16_kernel"           # blocks of 4x4 squares of 16x16
    assert name(desc(1, 16, 245, 32)) == "attn_block16_kernel"
    assert name(desc(1, 16, 245, 24)) == "attn_mfma_ragged_kernel"       # 24 is no multiple of 16 (nor does it divide 8)
    assert name(desc(1, 2, 100, 8, dtype=nb.NS_F32)) == "attn_generic_kernel"
    assert name(desc(1, 2, 24, 8, coords=True)) == "attn_mfma_ragged_kernel"
    assert name(desc(1, 2, 32, 16, coords=True)) == "attn_mfma_ragged_kernel"
    monkeypatch.setenv("NSATTN_KERNEL", "mfma")
    assert name(desc(2, 16, 128, 8)) == "attn_mfma_kernel"
    monkeypatch.setenv("NSATTN_KERNEL", "persist")
    assert name(desc(2, 16, 128, 8)) == "attn_mfma_persist_kernel"
    monkeypatch.setenv("NSATTN_KERNEL", "generic")
    assert name(desc(1, 16, 100, 8)) == "attn_generic_kernel"
    assert name(desc(2, 16, 128, 8)) == "attn_generic_kernel"
    monkeypatch.setenv("NSATTN_KERNEL", "block")
    assert name(desc(1, 2, 32, 16)) == "attn_block16_kernel"
    assert name(desc(2, 16, 128, 8)) != "attn_block16_kernel"           # a forced kernel that cannot serve falls back
    bad = desc(2, 16, 128, 8)
    bad.heads = 0
    assert name(bad) == ""


def _stack_desc(nb, keep_k, grid=128, block=8):
    d = nb.ns_vit_desc()
    a = d.block.attn
    a.batch, a.heads, a.head_dim = 1, 16, 64
    a.grid_h = a.grid_w = grid
    a.block, a.radius, a.n_global, a.dtype, a.tokens = block, 1, 1, nb.NS_BF16, 1 + grid * grid
    a.scale = 0.125
    d.block.dim, d.block.mlp_dim, d.block.ln_eps = 1024, 4096, 1e-6
    d.layers, d.prune_after, d.keep_k = 4, 2, keep_k
    return d


def test_stack_workspace_covers_the_pruned_blocks(nb):
    """A keep count within a few tokens of the grid size makes the blocks after the pruning stage need
    more workspace (token lists and counts) than the blocks on the full grid: the stack's workspace
    must cover both, for every proportion 0 <= p < 1 of the paper's pruning stage (keep_k = N is p = 0)."""
    N = 128 * 128
    for keep_k in (N, N - 1, N - 3, N - 100, (N * 60 + 99) // 100, 1):
        d = _stack_desc(nb, keep_k)
        total = nb.lib.vit_workspace_bytes(ctypes.byref(d))
        assert total > 0, nb.lib.ns_last_error()
        # the block on the pruned sequence, sized on its own
        pd = nb.ns_vit_block_desc()
        ctypes.memmove(ctypes.byref(pd), ctypes.byref(d.block), ctypes.sizeof(pd))
        pd.attn.tokens = 1 + keep_k
        pd.attn.coords = 0x1000          # never dereferenced on the host
        need_pruned = nb.lib.vit_block_workspace_bytes(ctypes.byref(pd))
        need_full = nb.lib.vit_block_workspace_bytes(ctypes.byref(d.block))
        assert need_pruned > 0 and need_full > 0
        no_prune = _stack_desc(nb, 0)
        base = nb.lib.vit_workspace_bytes(ctypes.byref(no_prune))
        # what the stack adds around a block does not depend on the block's workspace
        assert total - max(need_full, need_pruned) >= base - need_full - 4096
        assert total >= max(need_full, need_pruned)
    # the case that used to fall short: keep_k = N needs more than the full grid
    pd.attn.tokens = 1 + N
    assert nb.lib.vit_block_workspace_bytes(ctypes.byref(pd)) > nb.lib.vit_block_workspace_bytes(ctypes.byref(d.block))
