// C ABI of libnsattn.so: host-side validation and kernel dispatch.  No kernel lives here.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include "ns_common.h"
#include <algorithm>
#include <mutex>
#include <vector>

namespace ns {

static thread_local char g_err[512] = "";

ns_status fail(ns_status code, const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

ns_status check_launch(const char *what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(NS_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  return NS_OK;
}

int device_cu_count() {
  // (a function-local static is initialised once, thread-safely)
  static const int num_cus = [] {
    int dev = 0;
    hipDeviceProp_t prop;
    return (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
               ? prop.multiProcessorCount : 256;
  }();
  return num_cus;
}

ns_status reserve_lds_once(const void *kernel, int bytes) {
  static std::mutex mu;
  static std::vector<const void *> done;
  std::lock_guard<std::mutex> lock(mu);
  if (std::find(done.begin(), done.end(), kernel) != done.end()) return NS_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
    return fail(NS_ERR_HIP, "cannot reserve %d bytes of LDS", bytes);
  done.push_back(kernel);
  return NS_OK;
}

namespace {

inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline size_t elt_size(int dtype) { return dtype == NS_F32 ? 4 : 2; }

// Checks everything about a descriptor that does not involve the data pointers.
// need_grid = false (scoring): the grid fields and coords are not looked at.
ns_status validate_desc(const ns_attn_desc *d, bool need_out_strides, bool need_grid = true) {
  if (!d) return fail(NS_ERR_INVALID_ARG, "descriptor is NULL");
  if (d->batch < 1 || d->heads < 1 || d->head_dim < 1)
    return fail(NS_ERR_INVALID_ARG, "batch, heads and head_dim must be positive");
  if (d->n_global < 1) return fail(NS_ERR_INVALID_ARG, "n_global must be >= 1");
  if (need_grid && (d->grid_h < 1 || d->grid_w < 1 || d->block < 1 || d->radius < 0))
    return fail(NS_ERR_INVALID_ARG, "grid and block must be positive, radius >= 0");
  if (d->dtype != NS_F32 && d->dtype != NS_BF16)
    return fail(NS_ERR_INVALID_ARG, "dtype must be NS_F32 or NS_BF16");
  if (!(d->scale == d->scale) || d->scale - d->scale != 0.f)
    return fail(NS_ERR_INVALID_ARG, "scale must be finite");
  if (!need_grid) {
    if (d->tokens <= d->n_global) return fail(NS_ERR_INVALID_ARG, "tokens must exceed n_global");
  } else if (d->grid_h > 65535 || d->grid_w > 65535) {
    return fail(NS_ERR_INVALID_ARG, "grid sides must fit 16 bits");
  }
  const long long full = (long long)d->grid_h * d->grid_w + d->n_global;
  if (!need_grid) {
    // nothing more to check about the geometry
  } else if (full > 0x7fffffffLL) {
    return fail(NS_ERR_INVALID_ARG, "grid too large");
  } else if (d->coords == nullptr) {
    if (d->tokens != (int32_t)full)
      return fail(NS_ERR_INVALID_ARG, "tokens (%d) must equal n_global + grid_h*grid_w (%lld)",
                  d->tokens, full);
  } else {
    if (d->tokens <= d->n_global || d->tokens > (int32_t)full)
      return fail(NS_ERR_INVALID_ARG, "tokens (%d) out of range for a pruned sequence", d->tokens);
    if (!aligned(d->coords, 4)) return fail(NS_ERR_INVALID_ARG, "coords misaligned");
  }
  if (d->head_dim != 64) return fail(NS_ERR_UNSUPPORTED, "head_dim %d: only 64 is implemented", d->head_dim);
  if (need_grid && d->radius != 1)
    return fail(NS_ERR_UNSUPPORTED, "radius %d: only 1 (3x3 blocks) is implemented", d->radius);
  if (d->n_global > 256) return fail(NS_ERR_UNSUPPORTED, "more than 256 global tokens");
  if ((long long)d->heads * d->n_global > 1024)
    return fail(NS_ERR_UNSUPPORTED, "heads x n_global above 1024");
  if (need_grid && d->block > 256) return fail(NS_ERR_UNSUPPORTED, "block side above 256");
  const size_t es = elt_size(d->dtype);
  if (d->q_stride_t < d->head_dim || (d->q_stride_b * es) % 16 || (d->q_stride_h * es) % 16 ||
      (d->q_stride_t * es) % 16 || d->q_stride_b < 0 || d->q_stride_h < 0)
    return fail(NS_ERR_INVALID_ARG, "q/k/v strides must be non-negative, rows 16-byte aligned, stride_t >= head_dim");
  if (need_out_strides &&
      (d->out_stride_t < d->head_dim || (d->out_stride_b * es) % 16 || (d->out_stride_h * es) % 16 ||
       (d->out_stride_t * es) % 16 || d->out_stride_b < 0 || d->out_stride_h < 0))
    return fail(NS_ERR_INVALID_ARG, "out strides must be non-negative, rows 16-byte aligned, stride_t >= head_dim");
  return NS_OK;
}

struct AttnWorkspace {
  size_t partials_off, lists_off, counts_off, total;
};

// Per-block token lists are built for a pruned sequence and for a complete grid that the list
// kernel serves (bf16, head_dim 64, and either a block side other than 8 and 16 or a grid that the
// block side does not divide).
bool wants_lists(const ns_attn_desc &d) {
  return d.coords != nullptr || (!mfma_attn_supported(d) && ragged_attn_supported(d));
}

AttnWorkspace attn_workspace_layout(const ns_attn_desc &d) {
  AttnWorkspace w;
  size_t off = 0;
  w.partials_off = off;
  // (the sweep kernel leaves 4 records per row of blocks instead of one per 512 keys)
  const size_t nrec = std::max<size_t>(cls_num_chunks(d.tokens), d.block > 0 ? 4 * (size_t)((d.grid_h + d.block - 1) / d.block) : 0);
  off += align_up((size_t)d.batch * d.heads * d.n_global * nrec * kClsPartialFloats * 4, 256);
  w.lists_off = w.counts_off = off;
  if (wants_lists(d)) {
    const size_t nbh = (d.grid_h + d.block - 1) / d.block, nbw = (d.grid_w + d.block - 1) / d.block;
    off += align_up((size_t)d.batch * nbh * nbw * d.block * d.block * 4, 256);
    w.counts_off = off;
    off += align_up((size_t)d.batch * nbh * nbw * 4, 256);
  }
  w.total = off;
  return w;
}

ns_status check_workspace(void *ws, size_t have, size_t need) {
  if (need == 0) return NS_OK;
  if (!ws) return fail(NS_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
  if (!aligned(ws, 256)) return fail(NS_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (have < need) return fail(NS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
  return NS_OK;
}

}  // namespace
}  // namespace ns

using namespace ns;

extern "C" {

const char *ns_last_error(void) { return g_err; }
const char *ns_version(void) { return "0.1"; }

size_t ns_attn_workspace_bytes(const ns_attn_desc *desc) {
  if (validate_desc(desc, true) != NS_OK) return 0;
  return attn_workspace_layout(*desc).total;
}

// Kernel choice for the patch queries.  On the full grid with bf16, head_dim 64 and 8x8 or 16x16
// blocks there are three MFMA kernels that compute the same function: the sweep (8x8 blocks, also
// on grids that 8 does not divide; key tiles shared along a row of blocks, the global query's row
// computed on the way; wants at least one row of blocks per CU),
// the block kernel (block sides that are multiples of 16; key tiles shared by the four query tiles of
// a 16x16 square; wants two squares per CU), the persistent one-wave-per-SIMD kernel (needs two blocks per grid side), and the plain
// one-wave-per-query-tile kernel.  Every other bf16 problem with head_dim 64 (a pruned sequence, a
// grid that the block side does not divide, other block sides) takes the MFMA kernel that walks
// per-block token lists, and the rest (fp32, other head sizes) the fp32 FMA kernel.
// NSATTN_KERNEL = sweep | block | persist | mfma | lists | generic forces one of them where it applies.
enum PatchKernel { PK_SWEEP, PK_BLOCK16, PK_PERSIST, PK_MFMA, PK_RAGGED, PK_GENERIC };

static int device_cus() { return device_cu_count(); }

// (the environment is read once per call, here; the choice travels in AttnArgs::kernel)
static PatchKernel choose_patch_kernel(const ns_attn_desc &d) {
  const char *e = getenv("NSATTN_KERNEL");
  const char force = e ? e[0] : 0;
  if (force == 'g') return PK_GENERIC;        // serves every problem
  const bool tiled_ok = mfma_attn_supported(d);               // block side 8 or 16 dividing the grid
  const bool sweep_ok = sweep_attn_supported(d);              // block side 8, 4 or 2, any grid
  const bool block16_ok = block16_attn_supported(d);          // block side a multiple of 16, any grid
  const long long strips8 = (long long)d.batch * d.heads * ((d.grid_h + 7) / 8);   // the sweep's workgroups
  const long long squares16 = (long long)d.batch * d.heads * ((d.grid_h + 15) / 16) * ((d.grid_w + 15) / 16);   // the block kernel's
  if (force == 's' && sweep_ok) return PK_SWEEP;
  if (force == 'b' && block16_ok) return PK_BLOCK16;
  if (tiled_ok) {
    const bool persist_ok = persist_attn_supported(d);
    if (force == 'p' && persist_ok) return PK_PERSIST;
    if (force == 'm') return PK_MFMA;
    if (sweep_ok && strips8 >= device_cus()) return PK_SWEEP;
    if (block16_ok && squares16 >= 2LL * device_cus()) return PK_BLOCK16;
    if (persist_ok) return PK_PERSIST;
    return PK_MFMA;
  }
  // short edge blocks, 4x4 and 2x2 blocks: the sweep (and, for the former, the block kernel) takes them
  if (force != 'l' && sweep_ok && strips8 >= device_cus()) return PK_SWEEP;
  if (force != 'l' && block16_ok && squares16 >= 2LL * device_cus()) return PK_BLOCK16;
  if (ragged_attn_supported(d)) return PK_RAGGED;   // its lists: wants_lists()
  return PK_GENERIC;
}

static ns_status launch_patch_attention(const AttnArgs &a) {
  switch (a.kernel) {
    case PK_SWEEP: return launch_attn_sweep(a, nullptr, nullptr);
    case PK_BLOCK16: return launch_attn_block16(a);
    case PK_PERSIST: return launch_attn_persist(a);
    case PK_MFMA: return launch_attn_mfma(a);
    case PK_RAGGED: return launch_attn_ragged(a);
    default: return launch_attn_generic(a);
  }
}

// Shared by ns_attn_forward and the timing aid: validation, workspace carving, block lists.
static ns_status prepare_attn(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                              void *out, void *workspace, size_t workspace_bytes, void *stream,
                              AttnArgs &a, float *&partials, bool reuse_lists = false) {
  ns_status st = validate_desc(desc, true);
  if (st != NS_OK) return st;
  if (!q || !k || !v || !out) return fail(NS_ERR_INVALID_ARG, "q, k, v and out must not be NULL");
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(v, 16) || !aligned(out, 16))
    return fail(NS_ERR_INVALID_ARG, "q, k, v and out must be 16-byte aligned");
  if (out == q || out == k || out == v) return fail(NS_ERR_INVALID_ARG, "out must not alias an input");
  const ns_attn_desc &d = *desc;
  const AttnWorkspace w = attn_workspace_layout(d);
  st = check_workspace(workspace, workspace_bytes, w.total);
  if (st != NS_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  partials = reinterpret_cast<float *>(ws + w.partials_off);
  a.d = d; a.q = q; a.k = k; a.v = v; a.out = out; a.stream = s;
  BlockGeom &g = a.geom;
  g.grid_h = d.grid_h; g.grid_w = d.grid_w; g.block = d.block;
  g.nbh = (d.grid_h + d.block - 1) / d.block;
  g.nbw = (d.grid_w + d.block - 1) / d.block;
  g.n_global = d.n_global; g.tokens = d.tokens; g.cap = d.block * d.block;
  g.lists = nullptr; g.counts = nullptr;
  // (the workspace has room for lists whenever wants_lists(); a complete grid that the sweep serves
  // does without them)
  a.kernel = choose_patch_kernel(d);
  if (wants_lists(d) && (d.coords || a.kernel == PK_RAGGED)) {
    int32_t *lists = reinterpret_cast<int32_t *>(ws + w.lists_off);
    int32_t *counts = reinterpret_cast<int32_t *>(ws + w.counts_off);
    if (!reuse_lists) {
      st = d.coords ? launch_block_lists(d, lists, counts, s) : launch_grid_lists(d, lists, counts, s);
      if (st != NS_OK) return st;
    }
    g.lists = lists; g.counts = counts;
  }
  return NS_OK;
}

ns_status ns_attn_forward(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                          void *out, float *cls_logits, float *cls_lse, void *workspace,
                          size_t workspace_bytes, void *stream) {
  return attn_forward_impl(desc, q, k, v, out, cls_logits, cls_lse, nullptr, workspace, workspace_bytes, stream,
                           false);
}

ns_status ns_attn_forward_scores(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                                 void *out, float *cls_logits, float *cls_lse, float *scores,
                                 void *workspace, size_t workspace_bytes, void *stream) {
  if (!cls_logits || !scores) return fail(NS_ERR_INVALID_ARG, "cls_logits and scores must not be NULL");
  if (!aligned(scores, 4)) return fail(NS_ERR_INVALID_ARG, "scores misaligned");
  return attn_forward_impl(desc, q, k, v, out, cls_logits, cls_lse, scores, workspace, workspace_bytes, stream,
                           false);
}

}  // extern "C"

ns_status ns::attn_validate(const ns_attn_desc *desc) { return validate_desc(desc, true); }

ns_status ns::cls_scores_impl(const ns_attn_desc *desc, const void *q, const void *k, float *scores,
                              void *workspace, size_t workspace_bytes, void *stream) {
  ns_status st = validate_desc(desc, false, false);
  if (st != NS_OK) return st;
  if (!q || !k || !scores) return fail(NS_ERR_INVALID_ARG, "q, k and scores must not be NULL");
  if (!aligned(q, 16) || !aligned(k, 16) || !aligned(scores, 4))
    return fail(NS_ERR_INVALID_ARG, "q and k must be 16-byte aligned, scores 4-byte aligned");
  const ns_attn_desc &d = *desc;
  st = check_workspace(workspace, workspace_bytes, cls_scores_workspace_bytes(desc));
  if (st != NS_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(stream);
  float *logits = static_cast<float *>(workspace);
  float *partials = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) +
                                              align_up((size_t)d.batch * d.heads * d.n_global * d.tokens * 4, 256));
  st = launch_cls_row(d, q, k, nullptr, logits, partials, false, s);
  if (st != NS_OK) return st;
  return launch_cls_scores(d.batch, d.heads, d.tokens, d.n_global, logits, nullptr, partials,
                           cls_num_chunks(d.tokens), scores, s);
}

ns_status ns::attn_forward_impl(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                                void *out, float *cls_logits, float *cls_lse, float *scores, void *workspace,
                                size_t workspace_bytes, void *stream, bool reuse_lists) {
  if ((cls_logits && !aligned(cls_logits, 4)) || (cls_lse && !aligned(cls_lse, 4)))
    return fail(NS_ERR_INVALID_ARG, "cls_logits / cls_lse misaligned");
  AttnArgs a;
  float *partials = nullptr;
  ns_status st = prepare_attn(desc, q, k, v, out, workspace, workspace_bytes, stream, a, partials, reuse_lists);
  if (st != NS_OK) return st;
  const ns_attn_desc &d = a.d;
  if (a.kernel == PK_SWEEP && d.n_global == 1) {
    // this kernel computes the global query's partials and logits on the way
    st = launch_attn_sweep(a, cls_logits, partials);
    if (st != NS_OK) return st;
    if (scores) return launch_cls_combine_scores(d, partials, out, cls_lse, cls_logits, scores, a.stream, sweep_cls_chunks(d));
    return launch_cls_combine(d, partials, out, cls_lse, true, a.stream, sweep_cls_chunks(d));
  }
  st = launch_patch_attention(a);
  if (st != NS_OK) return st;
  // the global query's row: chunk partials, then the merge that also writes out[:, :, 0, :]
  st = launch_cls_row(d, q, k, v, cls_logits, partials, true, a.stream);
  if (st != NS_OK) return st;
  if (scores) return launch_cls_combine_scores(d, partials, out, cls_lse, cls_logits, scores, a.stream);
  return launch_cls_combine(d, partials, out, cls_lse, true, a.stream);
}

extern "C" {

ns_status ns_attn_patch_kernel_time(const ns_attn_desc *desc, const void *q, const void *k,
                                    const void *v, void *out, void *workspace,
                                    size_t workspace_bytes, int32_t reps, float *avg_ms,
                                    void *stream) {
  if (reps < 1 || !avg_ms) return fail(NS_ERR_INVALID_ARG, "reps must be positive and avg_ms not NULL");
  AttnArgs a;
  float *partials = nullptr;
  ns_status st = prepare_attn(desc, q, k, v, out, workspace, workspace_bytes, stream, a, partials);
  if (st != NS_OK) return st;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess)
    return fail(NS_ERR_HIP, "hipEventCreate failed");
  hipError_t e = hipEventRecord(e0, a.stream);
  const bool sweep = a.kernel == PK_SWEEP;
  for (int i = 0; i < reps && st == NS_OK; i++)
    st = sweep ? launch_attn_sweep(a, nullptr, partials) : launch_patch_attention(a);
  if (e == hipSuccess) e = hipEventRecord(e1, a.stream);
  if (e == hipSuccess) e = hipEventSynchronize(e1);
  float ms = 0.f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != NS_OK) return st;
  if (e != hipSuccess) return fail(NS_ERR_HIP, "event timing: %s", hipGetErrorString(e));
  *avg_ms = ms / (float)reps;
  return NS_OK;
}

const char *ns_attn_patch_kernel_name(const ns_attn_desc *desc) {
  if (validate_desc(desc, true) != NS_OK) return "";
  switch (choose_patch_kernel(*desc)) {
    case PK_SWEEP: return "attn_sweep_kernel";
    case PK_BLOCK16: return "attn_block16_kernel";
    case PK_PERSIST: return "attn_mfma_persist_kernel";
    case PK_MFMA: return "attn_mfma_kernel";
    case PK_RAGGED: return "attn_mfma_ragged_kernel";
    default: return "attn_generic_kernel";
  }
}

size_t cls_scores_workspace_bytes(const ns_attn_desc *desc) {
  if (validate_desc(desc, false, false) != NS_OK) return 0;
  const ns_attn_desc &d = *desc;
  return align_up((size_t)d.batch * d.heads * d.n_global * d.tokens * 4, 256) +
         align_up((size_t)d.batch * d.heads * d.n_global * cls_num_chunks(d.tokens) * kClsPartialFloats * 4, 256);
}

ns_status cls_scores(const ns_attn_desc *desc, const void *q, const void *k, float *scores,
                     void *workspace, size_t workspace_bytes, void *stream) {
  return cls_scores_impl(desc, q, k, scores, workspace, workspace_bytes, stream);
}

ns_status cls_scores_from_logits(int32_t batch, int32_t heads, int32_t tokens, int32_t n_global,
                                 const float *cls_logits, const float *cls_lse, float *scores,
                                 void *stream) {
  if (batch < 1 || heads < 1 || n_global < 1 || tokens <= n_global)
    return fail(NS_ERR_INVALID_ARG, "batch, heads, n_global must be positive and tokens > n_global");
  if ((long long)heads * n_global > 1024) return fail(NS_ERR_UNSUPPORTED, "heads x n_global above 1024");
  if (batch > 65535) return fail(NS_ERR_UNSUPPORTED, "batch above 65535");
  if (!cls_logits || !cls_lse || !scores) return fail(NS_ERR_INVALID_ARG, "NULL pointer");
  if (!aligned(cls_logits, 4) || !aligned(cls_lse, 4) || !aligned(scores, 4))
    return fail(NS_ERR_INVALID_ARG, "misaligned pointer");
  return launch_cls_scores(batch, heads, tokens, n_global, cls_logits, cls_lse, nullptr, 0, scores,
                           static_cast<hipStream_t>(stream));
}

size_t topk_filter_workspace_bytes(int32_t batch, int32_t n, int32_t k) {
  (void)k;
  if (batch < 1 || n < 1) return 0;
  return topk_select_workspace_bytes(batch, n);   // 0 for n <= 32768: the selection keeps its state in registers and LDS
}

ns_status topk_filter(int32_t batch, int32_t n, int32_t k, const float *scores, const void *x,
                      int32_t channels, int32_t x_dtype, const int32_t *coords_in,
                      int32_t *kept_idx, void *y, int32_t *coords_out, void *workspace,
                      size_t workspace_bytes, void *stream) {
  return topk_filter_global(batch, n, k, 1, scores, x, channels, x_dtype, coords_in, kept_idx, y, coords_out,
                            workspace, workspace_bytes, stream);
}

ns_status topk_filter_global(int32_t batch, int32_t n, int32_t k, int32_t n_global, const float *scores,
                             const void *x, int32_t channels, int32_t x_dtype, const int32_t *coords_in,
                             int32_t *kept_idx, void *y, int32_t *coords_out, void *workspace,
                             size_t workspace_bytes, void *stream) {
  if (batch < 1 || n < 1) return fail(NS_ERR_INVALID_ARG, "batch and n must be positive");
  if (n_global < 1) return fail(NS_ERR_INVALID_ARG, "n_global must be >= 1");
  if (k < 1 || k > n) return fail(NS_ERR_INVALID_ARG, "k = %d must be in [1, n = %d]", k, n);
  if (batch > 65535) return fail(NS_ERR_UNSUPPORTED, "batch above 65535");
  if (!scores || !kept_idx) return fail(NS_ERR_INVALID_ARG, "scores and kept_idx must not be NULL");
  if (!aligned(scores, 4) || !aligned(kept_idx, 4)) return fail(NS_ERR_INVALID_ARG, "misaligned pointer");
  if ((x == nullptr) != (y == nullptr)) return fail(NS_ERR_INVALID_ARG, "x and y must be given together");
  if ((coords_in == nullptr) != (coords_out == nullptr))
    return fail(NS_ERR_INVALID_ARG, "coords_in and coords_out must be given together");
  size_t row_bytes = 0;
  if (x) {
    if (x_dtype != NS_F32 && x_dtype != NS_BF16) return fail(NS_ERR_INVALID_ARG, "bad x_dtype");
    if (channels < 1) return fail(NS_ERR_INVALID_ARG, "channels must be positive");
    row_bytes = (size_t)channels * elt_size(x_dtype);
    if (row_bytes % 16) return fail(NS_ERR_UNSUPPORTED, "row size %zu bytes is not a multiple of 16", row_bytes);
    if (row_bytes / 16 > 0x7fffffffULL) return fail(NS_ERR_UNSUPPORTED, "row too long");
    if (!aligned(x, 16) || !aligned(y, 16)) return fail(NS_ERR_INVALID_ARG, "x and y must be 16-byte aligned");
    if (x == y) return fail(NS_ERR_INVALID_ARG, "y must not alias x");
  }
  const size_t need_ws = topk_select_workspace_bytes(batch, n);
  if (need_ws) {
    if (!workspace) return fail(NS_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need_ws);
    if (!aligned(workspace, 16)) return fail(NS_ERR_WORKSPACE, "workspace must be 16-byte aligned");
    if (workspace_bytes < need_ws)
      return fail(NS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need_ws);
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  ns_status st = launch_topk_select(batch, n, k, scores, coords_in, kept_idx, coords_out, workspace, s);
  if (st != NS_OK) return st;
  if (x) return launch_gather_rows(batch, n, k, n_global, row_bytes, x, kept_idx, y, s);
  return NS_OK;
}

}  // extern "C"
