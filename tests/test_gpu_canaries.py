"""Guard bands: every output and every workspace of the C ABI's calls sits between two 4 KB bands
of a byte pattern, the workspace exactly as large as the sizing call says; after the call the
bands must be untouched.  Catches writes before or beyond a buffer that parity on the buffer
itself cannot see."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2601_12150_amd import synth

pytestmark = pytest.mark.gpu

GUARD = 4096
PATTERN = 0xA5


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


class Guarded:
    """A device buffer of `nbytes` bytes with a band of PATTERN bytes on either side."""

    def __init__(self, nbytes):
        self.nbytes = int(nbytes)
        pad = (-self.nbytes) % 256
        self.raw = torch.full((GUARD + self.nbytes + pad + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        self.bytes = self.raw[GUARD:GUARD + self.nbytes]

    def view(self, dtype, shape):
        return self.bytes.view(dtype).view(shape)

    def intact(self):
        lo = self.raw[:GUARD]
        hi = self.raw[GUARD + self.nbytes:]
        return bool((lo == PATTERN).all()) and bool((hi == PATTERN).all())


def check(bands, what):
    torch.cuda.synchronize()
    for name, g in bands.items():
        assert g.intact(), "%s: bytes outside %s were written" % (what, name)


def attention_case(nb, monkeypatch, force, B, H, gh, gw, block, dtype, keep=None, n_global=1, seed=1):
    what = "attention %s B=%d H=%d grid=%dx%d block=%d %s keep=%s G=%d" % (force, B, H, gh, gw, block, dtype, keep, n_global)
    print(what, flush=True)
    if force:
        monkeypatch.setenv("NSATTN_KERNEL", force)
    else:
        monkeypatch.delenv("NSATTN_KERNEL", raising=False)
    q, k, v = synth.small_case(seed, B, H, 64, gh, gw, dtype, n_global=n_global)
    coords = None
    if keep is not None:
        rng = np.random.default_rng(seed)
        kept = np.sort(rng.choice(gh * gw, size=keep, replace=False))
        sel = np.concatenate([np.arange(n_global), n_global + kept])
        q, k, v = (np.ascontiguousarray(a[:, :, sel]) for a in (q, k, v))
        coords = torch.from_numpy(np.tile(synth.raster_coords(gh, gw)[kept], (B, 1))).cuda()
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    dq, dk, dv = (torch.from_numpy(a).to(tdt).cuda() for a in (q, k, v))
    T, G, elt = dq.shape[2], n_global, dq.element_size()
    bands = {"out": Guarded(B * H * T * 64 * elt), "logits": Guarded(B * H * G * T * 4), "lse": Guarded(B * H * G * 4),
             "scores": Guarded(B * (T - G) * 4)}
    out = bands["out"].view(tdt, (B, H, T, 64))
    desc = nb.make_desc(dq, gh, gw, block, None, out, coords, 1, n_global)
    nbytes = nb.lib.ns_attn_workspace_bytes(ctypes.byref(desc))
    assert nbytes > 0
    bands["workspace"] = Guarded(nbytes)
    print("  kernel", nb.lib.ns_attn_patch_kernel_name(ctypes.byref(desc)).decode(), "workspace", nbytes, flush=True)
    ptr = lambda g: ctypes.c_void_p(g.bytes.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    nb._check(nb.lib.ns_attn_forward_scores(ctypes.byref(desc), nb._ptr(dq), nb._ptr(dk), nb._ptr(dv), ptr(bands["out"]),
                                            ptr(bands["logits"]), ptr(bands["lse"]), ptr(bands["scores"]),
                                            ptr(bands["workspace"]), nbytes, stream))
    check(bands, what)
    assert bool(torch.isfinite(out.float()).all())
    # the same buffers through ns_attn_forward (no scores), and the standalone scoring
    nb._check(nb.lib.ns_attn_forward(ctypes.byref(desc), nb._ptr(dq), nb._ptr(dk), nb._ptr(dv), ptr(bands["out"]),
                                     ptr(bands["logits"]), ptr(bands["lse"]), ptr(bands["workspace"]), nbytes, stream))
    check(bands, what + " (forward)")
    if coords is None:
        n2 = nb.lib.cls_scores_workspace_bytes(ctypes.byref(desc))
        ws2 = Guarded(n2)
        nb._check(nb.lib.cls_scores(ctypes.byref(desc), nb._ptr(dq), nb._ptr(dk), ptr(bands["scores"]),
                                    ctypes.c_void_p(ws2.bytes.data_ptr()), n2, stream))
        bands["scoring workspace"] = ws2
        check(bands, what + " (cls_scores)")


@pytest.mark.parametrize("force,B,H,gh,gw,block,dtype", [
    ("sweep", 1, 2, 32, 32, 8, "bf16"), ("sweep", 2, 1, 20, 27, 8, "bf16"), ("sweep", 1, 2, 24, 24, 4, "bf16"),
    ("sweep", 1, 1, 19, 18, 2, "bf16"), ("block", 1, 2, 48, 48, 16, "bf16"), ("block", 1, 1, 40, 37, 16, "bf16"),
    ("block", 1, 1, 70, 70, 32, "bf16"), ("persist", 1, 2, 32, 32, 8, "bf16"), ("mfma", 1, 2, 16, 16, 8, "bf16"),
    ("lists", 1, 2, 21, 21, 7, "bf16"), ("generic", 1, 2, 12, 13, 4, "f32"), ("generic", 1, 1, 9, 9, 3, "bf16"),
    ("", 1, 16, 64, 64, 8, "bf16")])
def test_attention_writes_stay_inside_their_buffers(nb, monkeypatch, force, B, H, gh, gw, block, dtype):
    attention_case(nb, monkeypatch, force, B, H, gh, gw, block, dtype)


def test_pruned_and_multi_global_attention_writes_stay_inside(nb, monkeypatch):
    attention_case(nb, monkeypatch, "", 1, 2, 24, 24, 8, "bf16", keep=350)
    attention_case(nb, monkeypatch, "generic", 1, 2, 12, 12, 4, "f32", keep=77)
    attention_case(nb, monkeypatch, "", 1, 2, 16, 16, 8, "bf16", n_global=3)
    attention_case(nb, monkeypatch, "", 1, 2, 24, 24, 8, "bf16", keep=300, n_global=5)
    attention_case(nb, monkeypatch, "sweep", 1, 2, 20, 27, 8, "bf16", n_global=8)
    attention_case(nb, monkeypatch, "block", 1, 2, 37, 21, 16, "bf16", n_global=4)


@pytest.mark.parametrize("B,N,k,C", [(2, 1000, 377, 256), (3, 4096, 2458, 1024), (2, 16384, 9831, 64), (1, 20000, 7, 128),
                                     (1, 32768, 32768, 64), (2, 40000, 24000, 64), (1, 70001, 123, 64)])
def test_filter_writes_stay_inside_their_buffers(nb, B, N, k, C):
    what = "filter B=%d N=%d k=%d C=%d" % (B, N, k, C)
    print(what, flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(N + k)
    scores = torch.rand((B, N), device="cuda", generator=gen)
    x = torch.randn((B, 1 + N, C), device="cuda", generator=gen).to(torch.bfloat16)
    coords = torch.arange(B * N, dtype=torch.int32, device="cuda").view(B, N)
    nbytes = nb.lib.topk_filter_workspace_bytes(B, N, k)
    bands = {"kept": Guarded(B * k * 4), "y": Guarded(B * (1 + k) * C * 2), "coords_out": Guarded(B * k * 4),
             "workspace": Guarded(max(nbytes, 16))}
    kept, y, cout = nb.topk_filter(scores, k, x=x, coords=coords, kept_idx=bands["kept"].view(torch.int32, (B, k)),
                                   y=bands["y"].view(torch.bfloat16, (B, 1 + k, C)),
                                   coords_out=bands["coords_out"].view(torch.int32, (B, k)),
                                   workspace=bands["workspace"].bytes[:max(nbytes, 16)])
    check(bands, what)
    assert int(kept.min()) >= 0 and int(kept.max()) < N


def test_block_and_stack_writes_stay_inside_their_buffers(nb):
    B, g, blk, heads, dim, mlp, layers, after = 1, 24, 8, 8, 512, 640, 3, 1
    N, T = g * g, 1 + g * g
    keep = (N * 60 + 99) // 100
    rng = np.random.default_rng(3)
    x = torch.from_numpy(synth.round_to_bf16(rng.standard_normal((B, T, dim)).astype(np.float32))).to(torch.bfloat16).cuda()
    ws = [{kk: (torch.from_numpy(vv).to(torch.bfloat16) if kk.startswith("w_") else torch.from_numpy(vv)).cuda()
           for kk, vv in synth.make_block_weights(dim, mlp, seed=40 + i).items()} for i in range(layers)]
    # one block: workspace exactly as large as asked for
    d = nb.ns_vit_block_desc()
    a = d.attn
    a.batch, a.heads, a.head_dim, a.grid_h, a.grid_w, a.block, a.radius, a.n_global = B, heads, dim // heads, g, g, blk, 1, 1
    a.dtype, a.tokens, a.scale = nb.NS_BF16, T, float(dim // heads) ** -0.5
    d.dim, d.mlp_dim, d.ln_eps = dim, mlp, 1e-6
    nbytes = nb.lib.vit_block_workspace_bytes(ctypes.byref(d))
    bands = {"out": Guarded(B * T * dim * 2), "workspace": Guarded(nbytes)}
    out, scores = nb.vit_block_forward(x, ws[0], g, g, blk, heads, want_scores=True,
                                       out=bands["out"].view(torch.bfloat16, (B, T, dim)), workspace=bands["workspace"].bytes)
    check(bands, "vit_block_forward")
    # a stack with a pruning stage
    v = nb.ns_vit_desc()
    v.block = d
    v.layers, v.prune_after, v.keep_k = layers, after, keep
    nbytes = nb.lib.vit_workspace_bytes(ctypes.byref(v))
    bands = {"out": Guarded(B * (1 + keep) * dim * 2), "workspace": Guarded(nbytes)}
    out, kept = nb.vit_forward(x, ws, g, g, blk, heads, prune_after=after, keep_k=keep,
                               out=bands["out"].view(torch.bfloat16, (B, 1 + keep, dim)), workspace=bands["workspace"].bytes)
    check(bands, "vit_forward")
    assert bool(torch.isfinite(out.float()).all())
    # the same stack with two pruning stages
    after, keeps = [1, 2], [keep, keep // 3]
    aft = (ctypes.c_int32 * 2)(*after)
    kp = (ctypes.c_int32 * 2)(*keeps)
    nbytes = nb.lib.vit_stages_workspace_bytes(ctypes.byref(v), 2, aft, kp)
    bands = {"out": Guarded(B * (1 + keeps[-1]) * dim * 2), "workspace": Guarded(nbytes)}
    out, kept = nb.vit_forward_stages(x, ws, g, g, blk, heads, after, keeps,
                                      out=bands["out"].view(torch.bfloat16, (B, 1 + keeps[-1], dim)),
                                      workspace=bands["workspace"].bytes)
    check(bands, "vit_forward_stages")
    assert bool(torch.isfinite(out.float()).all()) and int(kept.max()) < N
