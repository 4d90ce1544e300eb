"""The library allocates nothing, clears nothing with memset calls and never synchronises, so its
launches can be recorded into a HIP graph.  A graph of the whole step (attention with the global
query's by-products, scores, selection, gather) and one of the block stack are replayed several
times, with eager work and synchronisations between the replays and new inputs in the same
buffers, and every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest
import torch

from paper_2601_12150_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nb():
    from paper_2601_12150_amd import binding
    return binding


def _bf16(a):
    return torch.from_numpy(a).to(torch.bfloat16).cuda()


@pytest.mark.parametrize("g,block,H", [(48, 8, 4), (132, 8, 2), (64, 16, 16)])
def test_step_graph_replays_match_eager(nb, g, block, H):
    B, D, C = 2, 64, 256
    N, T = g * g, 1 + g * g
    k = (N * 60 + 99) // 100
    rng = np.random.default_rng(g)
    q = torch.empty((B, H, T, D), dtype=torch.bfloat16, device="cuda")
    kk, v = torch.empty_like(q), torch.empty_like(q)
    x = torch.empty((B, T, C), dtype=torch.bfloat16, device="cuda")
    ws_sel = torch.empty(max(16, nb.lib.topk_filter_workspace_bytes(B, N, k)), dtype=torch.uint8, device="cuda")

    def fill(seed):
        a, b, c = synth.small_case(seed, B, H, D, g, g, "bf16")
        q.copy_(_bf16(a)); kk.copy_(_bf16(b)); v.copy_(_bf16(c))
        x.copy_(_bf16(np.random.default_rng(seed).standard_normal((B, T, C)).astype(np.float32)))

    def step():          # tensors the binding allocates while recording belong to the graph's pool
        out, logits, lse, scores = nb.ns_attn_forward_scores(q, kk, v, g, g, block, 0.125)
        kept, y, _ = nb.topk_filter(scores, k, x=x, workspace=ws_sel)
        return [out, logits, lse, scores, kept, y]

    fill(100)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # first calls set kernel attributes: not to be recorded
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        static = step()
    for r in range(3):
        fill(200 + r)                            # eager work between the replays: new inputs, same buffers
        want = step()
        torch.cuda.synchronize()
        for t in static:
            t.fill_(-1) if t.dtype == torch.int32 else t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b2 in zip(want, static):
            assert torch.equal(a, b2), "replay %d differs from the eager step" % r


def test_stack_graph_replays_match_eager(nb):
    B, g, block, heads, dim, mlp, layers = 1, 32, 8, 8, 512, 1024, 3
    N = g * g
    keep = (N * 60 + 99) // 100
    ws_blocks = []
    for i in range(layers):
        w = synth.make_block_weights(dim, mlp, seed=70 + i)
        ws_blocks.append({n: (_bf16(a) if a.ndim == 2 else torch.from_numpy(a).cuda()) for n, a in w.items()})
    x = torch.empty((B, 1 + N, dim), dtype=torch.bfloat16, device="cuda")

    def fill(seed):
        x.copy_(_bf16(synth.round_to_bf16(np.random.default_rng(seed).standard_normal((B, 1 + N, dim)).astype(np.float32))))

    def step():
        return nb.vit_forward(x, ws_blocks, g, g, block, heads, prune_after=1, keep_k=keep)

    fill(1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        out, kept = step()
    for r in range(3):
        fill(10 + r)
        want_out, want_kept = step()
        torch.cuda.synchronize()
        out.zero_(); kept.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(kept, want_kept) and torch.equal(out, want_out), "replay %d differs" % r
