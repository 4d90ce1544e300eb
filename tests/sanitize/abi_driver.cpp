// Walks the host side of the C ABI (argument validation, workspace sizing, kernel choice, error
// messages) without touching a GPU: every call below either only computes sizes or is refused on
// the host before anything is launched.  Built with -fsanitize=address,undefined on the host pass by
// tests/test_sanitizers_cpu.py.
#include <initializer_list>
#include <stdio.h>
#include <string.h>

#include "../../include/nsattn.h"

static int fails = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); fails++; } \
  } while (0)

static ns_attn_desc good(int grid, int block, int batch) {
  ns_attn_desc d;
  memset(&d, 0, sizeof(d));
  d.batch = batch; d.heads = 16; d.head_dim = 64;
  d.grid_h = d.grid_w = grid; d.block = block; d.radius = 1; d.n_global = 1; d.dtype = NS_BF16;
  d.tokens = 1 + grid * grid; d.scale = 0.125f;
  d.q_stride_t = 64; d.q_stride_h = (int64_t)d.tokens * 64; d.q_stride_b = d.q_stride_h * 16;
  d.out_stride_t = 64; d.out_stride_h = d.q_stride_h; d.out_stride_b = d.q_stride_b;
  return d;
}

int main() {
  void *fake = reinterpret_cast<void *>(0x10000), *fake2 = reinterpret_cast<void *>(0x20000);
  void *ws = reinterpret_cast<void *>(0x30000);
  // sizes and kernel names over the shapes of the workloads, with and without pruning
  const int grids[] = {28, 64, 128, 256, 100, 245, 8, 9, 1};
  const int blocks[] = {7, 8, 16, 64, 2, 4, 1, 256};
  for (int g : grids)
    for (int b : blocks) {
      ns_attn_desc d = good(g, b, 2);
      EXPECT(ns_attn_workspace_bytes(&d) > 0);
      EXPECT(strlen(ns_attn_patch_kernel_name(&d)) > 0);
      EXPECT(cls_scores_workspace_bytes(&d) > 0);
      d.coords = reinterpret_cast<const int32_t *>(0x1000);
      d.tokens = 1 + (g * g + 1) / 2;
      EXPECT(ns_attn_workspace_bytes(&d) > 0);
      d.dtype = NS_F32;
      EXPECT(ns_attn_workspace_bytes(&d) > 0);
    }
  // refused descriptors: nothing is launched, the message names the reason
  {
    ns_attn_desc d = good(16, 8, 1);
    d.tokens = 200;
    EXPECT(ns_attn_forward(&d, fake, fake, fake, fake2, nullptr, nullptr, ws, 1u << 30, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(strlen(ns_last_error()) > 0);
    d = good(16, 8, 1);
    d.head_dim = 32;
    EXPECT(ns_attn_forward(&d, fake, fake, fake, fake2, nullptr, nullptr, ws, 1u << 30, nullptr) == NS_ERR_UNSUPPORTED);
    d = good(16, 8, 1);
    EXPECT(ns_attn_forward(&d, fake, fake, fake, fake2, nullptr, nullptr, ws, 16, nullptr) == NS_ERR_WORKSPACE);
    EXPECT(ns_attn_forward(&d, fake, fake, fake, fake, nullptr, nullptr, ws, 1u << 30, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(ns_attn_forward_scores(&d, fake, fake, fake, fake2, nullptr, nullptr, nullptr, ws, 1u << 30, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(cls_scores(&d, fake, fake, nullptr, ws, 1u << 30, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(cls_scores(&d, fake, fake, reinterpret_cast<float *>(fake2), nullptr, 0, nullptr) == NS_ERR_WORKSPACE);
    EXPECT(cls_scores_from_logits(0, 16, 100, 1, nullptr, nullptr, nullptr, nullptr) == NS_ERR_INVALID_ARG);
    // the entry point with its own scratch memory refuses what does not fit, on the host
    d = good(700, 8, 1);
    EXPECT(cls_scores_workspace_bytes(&d) > cls_scores_static_max_bytes());
    EXPECT(cls_scores_static(&d, fake, fake, reinterpret_cast<float *>(fake2), nullptr) == NS_ERR_WORKSPACE);
  }
  // ranking and compaction
  {
    float *s = reinterpret_cast<float *>(fake);
    int32_t *kept = reinterpret_cast<int32_t *>(fake2);
    EXPECT(topk_filter(1, 100, 0, s, nullptr, 0, NS_BF16, nullptr, kept, nullptr, nullptr, nullptr, 0, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(topk_filter(1, 100, 101, s, nullptr, 0, NS_BF16, nullptr, kept, nullptr, nullptr, nullptr, 0, nullptr) == NS_ERR_INVALID_ARG);
    EXPECT(topk_filter(1, 100, 10, s, fake, 3, NS_BF16, nullptr, kept, ws, nullptr, nullptr, 0, nullptr) == NS_ERR_UNSUPPORTED);
    EXPECT(topk_filter(1, 100000, 10, s, nullptr, 0, NS_BF16, nullptr, kept, nullptr, nullptr, nullptr, 0, nullptr) == NS_ERR_WORKSPACE);
    EXPECT(topk_filter_workspace_bytes(1, 100, 10) == 0 && topk_filter_workspace_bytes(2, 32768, 100) == 0 && topk_filter_workspace_bytes(2, 32769, 100) > 0);
    EXPECT(topk_filter_global(1, 100, 10, 0, s, nullptr, 0, NS_BF16, nullptr, kept, nullptr, nullptr, nullptr, 0, nullptr) == NS_ERR_INVALID_ARG);
  }
  // transformer block and stack: sizes for every keep count around the grid size, refused shapes
  {
    ns_vit_desc v;
    memset(&v, 0, sizeof(v));
    v.block.attn = good(128, 8, 1);
    v.block.dim = 1024; v.block.mlp_dim = 4096; v.block.ln_eps = 1e-6f;
    v.layers = 24; v.prune_after = 12;
    const int N = 128 * 128;
    size_t last = 0;
    for (int keep : {0, 1, 9831, N - 100, N - 3, N - 1, N}) {
      v.keep_k = keep;
      const size_t t = vit_workspace_bytes(&v);
      EXPECT(t > 0);
      if (keep == N) EXPECT(t >= last);
      last = t;
    }
    v.keep_k = N + 1;
    EXPECT(vit_workspace_bytes(&v) == 0);
    v.keep_k = 100;
    EXPECT(vit_forward(&v, nullptr, fake, fake2, nullptr, ws, (size_t)1 << 40, nullptr) == NS_ERR_INVALID_ARG);
    {
      const int32_t after_ok[3] = {2, 5, 24}, keep_ok[3] = {9000, 9000, 10};
      const int32_t after_bad[2] = {5, 5}, keep_bad[2] = {10, 20};
      EXPECT(vit_stages_workspace_bytes(&v, 3, after_ok, keep_ok) > 0);
      EXPECT(vit_stages_workspace_bytes(&v, 0, nullptr, nullptr) > 0);
      EXPECT(vit_stages_workspace_bytes(&v, 2, after_bad, keep_ok) == 0);
      EXPECT(vit_stages_workspace_bytes(&v, 2, after_ok, keep_bad) == 0);
      EXPECT(vit_forward_stages(&v, 2, after_bad, keep_ok, nullptr, fake, fake2, nullptr, ws, (size_t)1 << 40, nullptr) == NS_ERR_INVALID_ARG);
      EXPECT(vit_forward_stages(&v, 3, after_ok, keep_ok, nullptr, fake, fake2, nullptr, ws, (size_t)1 << 40, nullptr) == NS_ERR_INVALID_ARG);
    }
    v.block.dim = 1000;      // heads * head_dim != dim
    EXPECT(vit_block_workspace_bytes(&v.block) == 0);
    EXPECT(vit_embed_workspace_bytes(1, 3, 128, 128, 16, 1024) > 0);
    EXPECT(vit_embed_workspace_bytes(1, 3, 128, 128, 16, 1000) == 0);
    EXPECT(linear_forward(100, 100, 64, fake, fake, reinterpret_cast<const float *>(fake), nullptr, 0, fake2, nullptr) == NS_ERR_UNSUPPORTED);
  }
  EXPECT(strcmp(ns_version(), "") != 0);
  if (fails) return 1;
  printf("C ABI sanitizer run ok\n");
  return 0;
}
