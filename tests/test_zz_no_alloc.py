"""cls_scores_static (the entry point that brings its own scratch memory) against cls_scores,
through the C ABI: same kernels, so the scores must agree bit for bit; two calls in a row, the
second on a smaller problem, so that what the first left in the shared buffer is in the way."""
import ctypes

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _scores_both_ways(nb, B, H, T, seed, G=1):
    g = torch.Generator(device="cpu").manual_seed(seed)
    q = torch.randn((B, H, T, 64), generator=g).to(torch.bfloat16).cuda()
    k = torch.randn((B, H, T, 64), generator=g).to(torch.bfloat16).cuda()
    desc = nb.make_desc(q, 1, T - G, 1, 0.125, None, None, 1, G)
    need = nb.lib.cls_scores_workspace_bytes(ctypes.byref(desc))
    assert 0 < need <= nb.lib.cls_scores_static_max_bytes()
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = torch.full((B, T - G), -1.0, dtype=torch.float32, device="cuda")
    out = torch.full((B, T - G), -2.0, dtype=torch.float32, device="cuda")
    st = nb.lib.cls_scores(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), ref.data_ptr(), ws.data_ptr(), need, None)
    assert st == nb.NS_OK, nb.lib.ns_last_error()
    st = nb.lib.cls_scores_static(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), out.data_ptr(), None)
    assert st == nb.NS_OK, nb.lib.ns_last_error()
    torch.cuda.synchronize()
    return ref.cpu().numpy(), out.cpu().numpy(), q, k


def test_static_scratch_entry_point_matches_cls_scores():
    from paper_2601_12150_amd import binding as nb
    import oracle
    # first call: 2 images x 16 heads x 16385 tokens (2.2 MB of the buffer); second: a smaller, ragged one
    for (B, H, T, seed) in ((2, 16, 16385, 11), (1, 4, 1000, 12)):
        ref, out, q, k = _scores_both_ways(nb, B, H, T, seed)
        assert np.array_equal(ref.view(np.uint32), out.view(np.uint32)), (B, H, T)
        assert np.isfinite(out).all() and (out > 0).all()
        if T <= 2000:   # and against the definition
            want = oracle.cls_scores(q.float().cpu().numpy(), k.float().cpu().numpy(), 0.125)
            assert np.allclose(out, want, rtol=5e-5, atol=1e-10)


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    from paper_2601_12150_amd import binding as nb
    T = 65537 * 4                       # 16 heads x 262148 logits x 4 B = 16.8 MB > 8 MiB
    q = torch.empty((1, 16, 1, 64), dtype=torch.bfloat16, device="cuda")
    desc = nb.make_desc(q, 1, 1, 1, 0.125, None, None, 1, 1)
    desc.tokens = T
    desc.q_stride_h = T * 64
    desc.q_stride_b = 16 * T * 64
    assert nb.lib.cls_scores_workspace_bytes(ctypes.byref(desc)) > nb.lib.cls_scores_static_max_bytes()
    fake = ctypes.c_void_p(0x10000)     # never dereferenced: the call is refused on the host
    st = nb.lib.cls_scores_static(ctypes.byref(desc), fake, fake, fake, None)
    assert st == nb.NS_ERR_WORKSPACE
    assert b"8388608" in nb.lib.ns_last_error()
