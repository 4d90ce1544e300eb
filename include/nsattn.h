/*
 * nsattn.h -- C ABI of libnsattn.so: neighbourhood-sparse ViT attention with a global
 * CLS token, CLS-score token ranking, top-k selection and sequence compaction for
 * AMD MI355X (gfx950).
 *
 * The operations follow the paper's Methodology section:
 *   "Memory-Efficiency Optimization"  -> ns_attn_forward, ns_attn_forward_scores
 *   "Time-Efficiency Optimization"    -> cls_scores, cls_scores_from_logits, topk_filter
 * and vit_block_forward wraps the attention in a pre-LayerNorm transformer block.
 *
 * Conventions that hold for every entry point
 *   - Token order: tokens 0..n_global-1 are global (CLS), token n_global + r*grid_w + c
 *     is the patch in grid row r, column c (raster order).
 *   - Every pointer except descriptor structs is a DEVICE pointer owned by the caller.
 *     The library never allocates, frees or synchronises; every call enqueues its kernels
 *     on `stream` (a hipStream_t passed as void*, NULL = the default stream) and returns.
 *   - Scratch memory is passed in as `workspace`; `*_workspace_bytes` tells how much a call
 *     with the same arguments needs.  Workspace pointers must be 256-byte aligned.
 *   - Arguments are validated on the host before anything is launched: a call that returns
 *     an error has launched nothing and written nothing.  Outputs must not alias inputs.
 *   - Results are deterministic: no floating-point atomics, fixed reduction orders.
 *   - Return value: NS_OK or an error code; ns_last_error() gives a message for the last
 *     error on the calling thread.
 */
#ifndef NSATTN_H
#define NSATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NS_OK = 0,
  NS_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, k out of range, ...        */
  NS_ERR_UNSUPPORTED = 2, /* well-formed but not implemented (e.g. head_dim != 64)       */
  NS_ERR_WORKSPACE = 3,   /* workspace missing, misaligned or too small                  */
  NS_ERR_HIP = 4          /* a HIP runtime call or a kernel launch failed                */
} ns_status;

typedef enum { NS_F32 = 0, NS_BF16 = 1 } ns_dtype;

/*
 * Shape of one attention call.
 *
 * Pattern (paper, "Memory-Efficiency Optimization"): the patch grid is cut into
 * block x block token blocks (the paper's "window size"); a patch query attends to the
 * patches of the (2*radius+1)^2 blocks around its own block, clipped at the image edge
 * (no wrap-around, no padding keys), and to the global tokens; a global query attends to
 * every token.  The last block of a row/column is short when the grid is not divisible.
 *
 * q, k, v share one set of element strides and out has its own, so q/k/v may be views of
 * a fused [B,T,3,H,D] projection and out a [B,T,H,D] tensor.  The head_dim axis is
 * contiguous.  Rows must be 16-byte aligned (base pointers and strides*elt multiples of 16).
 *
 * coords == NULL: the sequence is the full grid, tokens == n_global + grid_h*grid_w.
 * coords != NULL (after pruning): device array [batch, tokens - n_global] holding the
 * original grid position (r << 16 | c) of each surviving patch token; positions must be
 * distinct within an image and inside the grid.  The mask is evaluated on those original
 * positions.  This precondition is the caller's: the positions live in device memory and no
 * call checks them.  A token whose position lies outside the grid, or one of several tokens
 * that claim the same position beyond what a block holds, belongs to no block: no key set is
 * defined for it, its row of out is left as it was, and the call still returns NS_OK.  The
 * coords_out that topk_filter and gather write from valid coords_in always satisfy it.
 */
typedef struct ns_attn_desc {
  int32_t batch;     /* B >= 1                                                           */
  int32_t heads;     /* H >= 1                                                           */
  int32_t head_dim;  /* D; this build implements 64                                      */
  int32_t grid_h;    /* patch grid rows                                                  */
  int32_t grid_w;    /* patch grid columns                                               */
  int32_t block;     /* b >= 1: side of a token block                                    */
  int32_t radius;    /* neighbourhood radius in blocks; this build implements 1 (3x3)    */
  int32_t n_global;  /* G >= 1 leading global tokens (CLS, registers); G <= 256, H*G <= 1024 */
  int32_t dtype;     /* ns_dtype of q, k, v, out; accumulation is always fp32            */
  int32_t tokens;    /* T: tokens present per image                                      */
  float scale;       /* logit multiplier, normally 1/sqrt(D)                             */
  int64_t q_stride_b, q_stride_h, q_stride_t;     /* element strides of q, k and v       */
  int64_t out_stride_b, out_stride_h, out_stride_t; /* element strides of out            */
  const int32_t *coords; /* NULL or device [B, T - G]                                    */
} ns_attn_desc;

/* Bytes of workspace ns_attn_forward needs for this descriptor (0 on an invalid one). */
size_t ns_attn_workspace_bytes(const ns_attn_desc *desc);

/*
 * Masked softmax attention for all T query tokens.
 *   q, k, v   in   [B,H,T,D] by the descriptor's q strides, dtype desc->dtype
 *   out       out  [B,H,T,D] by the descriptor's out strides, same dtype
 *   cls_logits out, nullable  [B,H,G,T] fp32: scale * <q_g, k_j> for global query g
 *   cls_lse    out, nullable  [B,H,G]   fp32: log(sum_j exp(cls_logits[g][j])) (natural log)
 * cls_logits and cls_lse are by-products of the global queries' rows; passing them lets
 * cls_scores_from_logits produce the importance scores without reading K again.
 * Several global tokens (paper, "Memory-Efficiency Optimization": a few designated global
 * tokens attend to, and are attended by, every token): each of the G global queries sees
 * all T keys, and every patch query sees the G global keys besides its neighbourhood.
 */
ns_status ns_attn_forward(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                          void *out, float *cls_logits, float *cls_lse, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * ns_attn_forward followed by cls_scores_from_logits (paper, "Time-Efficiency Optimization": the
 * importance of a patch is the attention the global tokens pay to it, averaged over heads), with
 * the merge of the global queries' rows and the scoring in one launch.
 *   cls_logits out, required  [B,H,G,T] fp32 (the scoring reads it back)
 *   cls_lse    out, nullable  [B,H,G]
 *   scores     out, required  [B, T-G] fp32
 * Everything else as in ns_attn_forward.
 */
ns_status ns_attn_forward_scores(const ns_attn_desc *desc, const void *q, const void *k, const void *v,
                                 void *out, float *cls_logits, float *cls_lse, float *scores,
                                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * Importance scores (paper, "Time-Efficiency Optimization": a score per token derived from
 * the global attention weights).  scores[b, j] = mean over heads and over the G global
 * queries of the softmax weight that the global query puts on patch key G + j, the softmax
 * running over all T keys.
 * Only batch, heads, head_dim, n_global, tokens, dtype, scale and the q strides of the
 * descriptor are used.
 *   q, k    in   as in ns_attn_forward (only tokens 0..G-1 of q are read)
 *   scores  out  [B, T-G] fp32
 */
size_t cls_scores_workspace_bytes(const ns_attn_desc *desc);
ns_status cls_scores(const ns_attn_desc *desc, const void *q, const void *k, float *scores,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * cls_scores for callers that cannot allocate device memory or pass a workspace: code recorded
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as cls_scores (same kernels), but the scratch memory is a buffer inside the library
 * (cls_scores_static_max_bytes() bytes per GPU, 8 MiB, held until the process ends).  The call
 * allocates and frees nothing.  A problem whose cls_scores_workspace_bytes exceeds the buffer is
 * rejected with NS_ERR_WORKSPACE before anything is launched.  All calls on one GPU share the
 * buffer: calls that may overlap in time on the same GPU (different streams, different threads)
 * race and must be serialised by the caller; calls on one stream are ordered and safe.
 */
size_t cls_scores_static_max_bytes(void);
ns_status cls_scores_static(const ns_attn_desc *desc, const void *q, const void *k, float *scores, void *stream);

/* The same scores from ns_attn_forward's by-products: logits [B,H,G,T], lse [B,H,G]. */
ns_status cls_scores_from_logits(int32_t batch, int32_t heads, int32_t tokens, int32_t n_global,
                                 const float *cls_logits, const float *cls_lse, float *scores,
                                 void *stream);

/*
 * Ranking and compaction (paper, "Time-Efficiency Optimization": rank all tokens, discard
 * the lowest-scoring proportion, shorten the sequence for the following layers).
 * Keeps the k highest-scoring of N patch tokens per image; equal scores rank by lower
 * index first (-0.0 == +0.0); scores must not be NaN.
 *   scores     in   [B,N] fp32
 *   x          in, nullable   [B, 1+N, C] token-major activations, dtype x_dtype
 *   coords_in  in, nullable   [B,N] int32 grid positions (r << 16 | c)
 *   kept_idx   out  [B,k] int32, patch indices 0..N-1 in ascending order
 *   y          out, nullable (required iff x given) [B, 1+k, C]: row 0 = x row 0 (CLS),
 *              row 1+t = x row 1+kept_idx[t]; bit copies.  C*elt must be a multiple of 16.
 *   coords_out out, nullable (required iff coords_in given) [B,k]
 *   workspace  device scratch of topk_filter_workspace_bytes(batch, n, k) bytes, 16-byte aligned
 *              (0 bytes for n <= 32768: NULL is accepted then); NS_ERR_WORKSPACE if missing or short.
 *              Rows longer than that are selected by several workgroups per image, which exchange
 *              digit histograms through it between launches.
 */
size_t topk_filter_workspace_bytes(int32_t batch, int32_t n, int32_t k);
ns_status topk_filter(int32_t batch, int32_t n, int32_t k, const float *scores, const void *x,
                      int32_t channels, int32_t x_dtype, const int32_t *coords_in,
                      int32_t *kept_idx, void *y, int32_t *coords_out, void *workspace,
                      size_t workspace_bytes, void *stream);
/* The same with n_global leading global rows instead of one: x [B, G+N, C], y [B, G+k, C],
 * rows 0..G-1 copied, row G+t = x row G+kept_idx[t]. */
ns_status topk_filter_global(int32_t batch, int32_t n, int32_t k, int32_t n_global, const float *scores,
                             const void *x, int32_t channels, int32_t x_dtype, const int32_t *coords_in,
                             int32_t *kept_idx, void *y, int32_t *coords_out, void *workspace,
                             size_t workspace_bytes, void *stream);

/*
 * One pre-LayerNorm transformer block around the sparse attention:
 *   h = x + Wproj * Attn(LN1(x)) + bproj;   y = h + W2 * gelu(W1 * LN2(h) + b1) + b2
 * with gelu the exact (erf) form.  Activations and weights are bf16, LayerNorm parameters
 * and biases fp32; every GEMM accumulates in fp32.
 * Weight layout: row-major [out_features, in_features] (y = x * W^T + b).
 * attn describes the attention (its strides are ignored: the block lays q/k/v out itself);
 * attn.heads * attn.head_dim must equal dim.
 *   x_in  in  [B,T,dim] bf16;  x_out out [B,T,dim] bf16 (may not alias x_in)
 *   scores_out out, nullable [B, T-G] fp32: the importance scores of this block's attention
 */
typedef struct ns_vit_block_desc {
  ns_attn_desc attn;
  int32_t dim;      /* model width, heads*head_dim */
  int32_t mlp_dim;  /* hidden width of the MLP     */
  float ln_eps;
} ns_vit_block_desc;

typedef struct ns_vit_block_weights {
  const float *ln1_g, *ln1_b;   /* [dim]                     */
  const void *w_qkv;            /* bf16 [3*dim, dim]: rows 0..dim-1 -> q, then k, then v */
  const float *b_qkv;           /* [3*dim]                   */
  const void *w_proj;           /* bf16 [dim, dim]           */
  const float *b_proj;          /* [dim]                     */
  const float *ln2_g, *ln2_b;   /* [dim]                     */
  const void *w_fc1;            /* bf16 [mlp_dim, dim]       */
  const float *b_fc1;           /* [mlp_dim]                 */
  const void *w_fc2;            /* bf16 [dim, mlp_dim]       */
  const float *b_fc2;           /* [dim]                     */
} ns_vit_block_weights;

size_t vit_block_workspace_bytes(const ns_vit_block_desc *desc);
ns_status vit_block_forward(const ns_vit_block_desc *desc, const ns_vit_block_weights *weights,
                            const void *x_in, void *x_out, float *scores_out, void *workspace,
                            size_t workspace_bytes, void *stream);

/*
 * One linear map of the block with its fused epilogue, exposed on its own for tests and
 * measurement (the block applies it four times: QKV, attention projection, the two MLP layers of
 * the standard ViT block the paper builds on):
 *     y[m][n] = act( sum_k x[m][k] * w[n][k] + bias[n] ) + residual[m][n]
 *   x        in  [M, K] bf16, row-major          w     in  [N, K] bf16 (out-features major)
 *   bias     in  [N] fp32                        residual in, nullable [M, N] bf16
 *   gelu     non-zero: act = exact (erf) GELU, else identity
 *   y        out [M, N] bf16; must not alias x, w or residual
 * fp32 accumulation, one rounding to bf16 at the end.  N must be a multiple of 128 and K of 64
 * (NS_ERR_UNSUPPORTED otherwise); all pointers 16-byte aligned.  No workspace.
 */
ns_status linear_forward(int32_t M, int32_t N, int32_t K, const void *x, const void *w, const float *bias,
                         const void *residual, int32_t gelu, void *y, void *stream);

/*
 * A stack of `layers` such blocks with one pruning stage (paper, "Time-Efficiency Optimization":
 * the pruning is applied once, after several initial layers, and shortens the sequence for all
 * subsequent layers).  Blocks 0 .. prune_after-1 run on the full grid; the importance scores of
 * block prune_after-1's attention select keep_k patches per image (topk_filter); the remaining
 * blocks run on [CLS; kept patches] with the mask evaluated on the kept patches' original grid
 * positions.  prune_after == 0 or keep_k == 0 disables pruning.
 *   block       shape of every block; block.attn describes the full grid (coords must be NULL)
 *   weights     HOST array [layers] of per-block device weight pointers
 *   x_in   in   [B, T, dim] bf16
 *   x_out  out  [B, 1 + keep_k, dim] bf16 with pruning, else [B, T, dim]
 *   kept_idx out, nullable [B, keep_k] int32: the kept patch indices, ascending
 */
typedef struct ns_vit_desc {
  ns_vit_block_desc block;
  int32_t layers;
  int32_t prune_after;
  int32_t keep_k;
} ns_vit_desc;

size_t vit_workspace_bytes(const ns_vit_desc *desc);
ns_status vit_forward(const ns_vit_desc *desc, const ns_vit_block_weights *weights, const void *x_in,
                      void *x_out, int32_t *kept_idx, void *workspace, size_t workspace_bytes,
                      void *stream);

/*
 * The same stack, also handing out the patch tokens after chosen blocks as spatial feature maps
 * (paper, "Segmentation": the segmentation head needs feature maps that preserve the image's
 * spatial structure, so the sparse attention runs in every layer and nothing is pruned before a
 * map is taken).  Tokens are never permuted inside the library, so a map is simply the patch rows
 * in raster order.
 *   n_taps      number of feature maps (0: identical to vit_forward)
 *   tap_layers  HOST array [n_taps], ascending, 1-based: map i is taken after block tap_layers[i];
 *               with a pruning stage every tap must lie at or before prune_after
 *   tap_out     HOST array [n_taps] of device pointers, each [B, grid_h*grid_w, dim] bf16
 */
ns_status vit_forward_features(const ns_vit_desc *desc, const ns_vit_block_weights *weights, const void *x_in,
                               void *x_out, int32_t *kept_idx, int32_t n_taps, const int32_t *tap_layers,
                               void *const *tap_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The stack with several pruning stages instead of one: stage i follows block stage_after[i] and keeps
 * stage_keep[i] of the patches still present, ranked by that block's importance scores (the scores of a
 * pruned sequence are those of its own tokens: softmax over the tokens present).  The paper describes a
 * single stage ("Time-Efficiency Optimization"); this entry point applies its selection rule repeatedly.
 * desc->prune_after and desc->keep_k are ignored.
 *   stage_after  HOST array [n_stages], 1-based block numbers, strictly ascending
 *   stage_keep   HOST array [n_stages], positive, stage_keep[0] <= patches, never growing
 *   x_out  out   [B, G + stage_keep[n_stages-1], dim] bf16 (n_stages == 0: [B, T, dim])
 *   kept_idx out, nullable [B, stage_keep[n_stages-1]] int32: ORIGINAL patch indices of the final
 *                survivors, ascending
 *   workspace    vit_stages_workspace_bytes(...) bytes, 256-byte aligned
 * NS_ERR_INVALID_ARG for stage lists that break the rules above.
 */
size_t vit_stages_workspace_bytes(const ns_vit_desc *desc, int32_t n_stages, const int32_t *stage_after,
                                  const int32_t *stage_keep);
ns_status vit_forward_stages(const ns_vit_desc *desc, int32_t n_stages, const int32_t *stage_after,
                             const int32_t *stage_keep, const ns_vit_block_weights *weights, const void *x_in,
                             void *x_out, int32_t *kept_idx, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Tokenisation of the ViT backbone the blocks belong to (paper, "Settings": a ViT foundation model
 * is the backbone; its input is the resized image): non-overlapping patch x patch pixel squares, one
 * linear map per patch, a learned CLS token in front, learned position embeddings added.
 *     x_out[b, 0, :]     = cls_token + pos_embed[0, :]
 *     x_out[b, 1 + n, :] = w_patch . pixels(patch n of image b) + b_patch + pos_embed[1 + n, :]
 * with patch n = (row n / grid_w, column n % grid_w) of the patch grid and the pixels of a patch in
 * the order (channel, y, x), x fastest (the layout of a convolution weight [dim, channels, patch, patch]).
 *   pixels     in  [B, channels, grid_h*patch, grid_w*patch] bf16
 *   w_patch    in  [dim, channels*patch*patch] bf16         b_patch  in  [dim] fp32
 *   cls_token  in  [dim] bf16                               pos_embed in [1 + grid_h*grid_w, dim] bf16
 *   x_out      out [B, 1 + grid_h*grid_w, dim] bf16 (the x_in of vit_forward)
 * fp32 accumulation, one rounding to bf16.  dim must be a multiple of 128.  w_patch, b_patch,
 * pos_embed and x_out 16-byte aligned; workspace of vit_embed_workspace_bytes bytes, 256-byte aligned.
 */
size_t vit_embed_workspace_bytes(int32_t batch, int32_t channels, int32_t grid_h, int32_t grid_w, int32_t patch,
                                 int32_t dim);
ns_status vit_embed(int32_t batch, int32_t channels, int32_t grid_h, int32_t grid_w, int32_t patch, int32_t dim,
                    const void *pixels, const void *w_patch, const float *b_patch, const void *cls_token,
                    const void *pos_embed, void *x_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aid for benchmarks (not part of the method): enqueues `reps` launches of the
 * patch-query attention kernel alone (the dominant kernel of ns_attn_forward; no CLS row)
 * on `stream`, bracketed by HIP events recorded on that stream, WAITS for them, and stores
 * the average duration of one launch in milliseconds in *avg_ms (a HOST pointer).  The only
 * entry point that synchronises.  Arguments as in ns_attn_forward; out rows of patch tokens
 * are written, row 0 is not.
 */
ns_status ns_attn_patch_kernel_time(const ns_attn_desc *desc, const void *q, const void *k,
                                    const void *v, void *out, void *workspace,
                                    size_t workspace_bytes, int32_t reps, float *avg_ms,
                                    void *stream);

/*
 * Name of the kernel that ns_attn_forward launches for the patch queries of `desc` on the current
 * device (the one ns_attn_patch_kernel_time measures); "" for an invalid descriptor.  Host only,
 * launches nothing.
 */
const char *ns_attn_patch_kernel_name(const ns_attn_desc *desc);

/* Message for the last error returned on this thread (static storage; never free it). */
const char *ns_last_error(void);

/* Library version, "major.minor". */
const char *ns_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NSATTN_H */
