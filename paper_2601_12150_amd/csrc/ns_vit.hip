// Pre-LayerNorm transformer block around the neighbourhood-sparse attention (gfx950):
//   h = x + Wproj Attn(LN1 x) + bproj;   y = h + W2 gelu(W1 LN2 h + b1) + b2
// The paper applies its sparse attention and its token pruning inside a ViT backbone
// ("Experimental Setups": UNI-2); this file supplies that surrounding block so that the path can
// be run and measured end to end: a LayerNorm kernel, one bf16 MFMA GEMM kernel with fused
// epilogues (bias, exact GELU, residual), and the host-side sequencing.
#include "ns_common.h"

namespace ns {

namespace {

// ------------------------------------------------------------------------------------------
// LayerNorm: one wave per token row, fp32 statistics, bf16 in/out, fp32 gamma/beta.
// Bound: HBM (reads and writes each element once).
// ------------------------------------------------------------------------------------------
template <int VPL>   // 8-element vectors per lane: dim = 512 * VPL
__global__ __launch_bounds__(256) void layernorm_kernel(const uint16_t *x, const float *gamma,
                                                        const float *beta, uint16_t *y, int rows,
                                                        float eps) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= rows) return;
  constexpr int DIM = 512 * VPL;
  const uint16_t *xr = x + (size_t)row * DIM;
  float v[VPL][8];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < VPL; i++) {
    const uint4 u = *reinterpret_cast<const uint4 *>(xr + (i * 64 + lane) * 8);
    v[i][0] = bf16_lo(u.x); v[i][1] = bf16_hi(u.x); v[i][2] = bf16_lo(u.y); v[i][3] = bf16_hi(u.y);
    v[i][4] = bf16_lo(u.z); v[i][5] = bf16_hi(u.z); v[i][6] = bf16_lo(u.w); v[i][7] = bf16_hi(u.w);
#pragma unroll
    for (int e = 0; e < 8; e++) s += v[i][e];
  }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) s += __shfl_xor(s, off);
  const float mean = s * (1.f / DIM);
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < VPL; i++)
#pragma unroll
    for (int e = 0; e < 8; e++) { const float d = v[i][e] - mean; q = __builtin_fmaf(d, d, q); }
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) q += __shfl_xor(q, off);
  const float rstd = 1.f / __builtin_sqrtf(q * (1.f / DIM) + eps);
  uint16_t *yr = y + (size_t)row * DIM;
#pragma unroll
  for (int i = 0; i < VPL; i++) {
    const int c = (i * 64 + lane) * 8;
    const f32x4 g0 = *reinterpret_cast<const f32x4 *>(gamma + c), g1 = *reinterpret_cast<const f32x4 *>(gamma + c + 4);
    const f32x4 b0 = *reinterpret_cast<const f32x4 *>(beta + c), b1 = *reinterpret_cast<const f32x4 *>(beta + c + 4);
    float o[8];
#pragma unroll
    for (int e = 0; e < 4; e++) {
      o[e] = __builtin_fmaf((v[i][e] - mean) * rstd, g0[e], b0[e]);
      o[4 + e] = __builtin_fmaf((v[i][4 + e] - mean) * rstd, g1[e], b1[e]);
    }
    uint4 u = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]), pack_bf16(o[4], o[5]), pack_bf16(o[6], o[7])};
    *reinterpret_cast<uint4 *>(yr + c) = u;
  }
}

// ------------------------------------------------------------------------------------------
// GEMM: C[m][n] = sum_k A[m][k] * W[n][k] + bias[n], optional exact GELU, optional residual
// R[m][n]; A, W, R, C bf16 (row-major, k contiguous for both operands), bias fp32, fp32 accumulate.
// Bound: bf16 MFMA; 2*M*N*K FLOP.
//
// Workgroup tile 128 (m) x 128 (n), k-step 64; 4 waves, each a 64x64 quadrant = 2x2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16.  The product is formed transposed (W rows as the A operand, token
// rows as the B operand) so that a lane ends up with 4 consecutive n of one token row per
// register group: 8-byte stores, and bias / residual in the same layout.  Both operand tiles
// go global -> LDS by direct 16-byte transfers (no registers), double-buffered, XOR-swizzled
// (16-byte chunk c of row r sits at chunk c ^ ((r>>1)&7)) so that the per-lane 16-byte
// fragment reads are free of bank conflicts.
// ------------------------------------------------------------------------------------------
struct GemmParams {
  const uint16_t *a, *w, *r;
  const float *bias;
  uint16_t *c;
  int M, N, K;
  int gelu;
};


typedef bf16x8 __attribute__((address_space(3))) *lds_bf16x8_ptr;


__global__ __launch_bounds__(256, 2) void gemm_bf16_kernel(GemmParams p) {
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;          // quadrant of this wave
  // consecutive workgroups walk n first, so the workgroups that share a token tile run together
  const int ntn = p.N / 128;
  const int bm = blockIdx.x / ntn, bn = blockIdx.x % ntn;
  const int m0 = bm * 128, n0 = bn * 128;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];   // [stage][A 16K | W 16K]
  const uint32_t lds0 = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);

  // ---- transfers: a 128-row x 64-k tile is 16 requests of 8 rows; this wave issues 4 of the
  // token tile and 4 of the weight tile.  Slot `lane` of request `it` is row it*8 + lane/8,
  // physical chunk lane%8, logical chunk (lane%8) ^ ((row>>1)&7).
  const char *ab = reinterpret_cast<const char *>(p.a);
  const char *wb = reinterpret_cast<const char *>(p.w);
  const uint32_t rowB = (uint32_t)p.K * 2u;
  uint32_t aoff[4], woff[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    const int it = wave * 4 + j, row = it * 8 + (lane >> 3);
    const int chunk = (lane & 7) ^ ((row >> 1) & 7);
    const int am = min(m0 + row, p.M - 1);            // rows past M repeat the last row (never stored)
    aoff[j] = (uint32_t)am * rowB + 16u * chunk;
    woff[j] = (uint32_t)(n0 + row) * rowB + 16u * chunk;
  }
  auto issue = [&](int kt, int stage) {
    const char *ak = ab + (size_t)kt * 128, *wk = wb + (size_t)kt * 128;
    const uint32_t base = lds0 + stage * 32768 + wave * 4 * 1024;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      dma16(ak, aoff[j], base + j * 1024);
      dma16(wk, woff[j], base + 16384 + j * 1024);
    }
  };
  // ---- fragment reads: lane (row l32 [+32], half hh) reads logical chunks 4*hh + ks
  unsigned char *frd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ks++) frd[ks] = smem + l32 * 128 + 16 * ((4 * hh + ks) ^ ((l32 >> 1) & 7));

  f32x16 acc[2][2];   // [nt (weight rows)][mt (token rows)]: rows n, column m
#pragma unroll
  for (int i = 0; i < 2; i++)
#pragma unroll
    for (int j = 0; j < 2; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  const int nk = p.K / 64;
  issue(0, 0);
  for (int kt = 0; kt < nk; kt++) {
    const int stage = kt & 1;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's share of tile kt has landed
    __syncthreads();                                    // everyone's has; everyone is done with tile kt-1
    if (kt + 1 < nk) issue(kt + 1, stage ^ 1);
    bf16x8 fa[2][4], fw[2][4];
#pragma unroll
    for (int t = 0; t < 2; t++)
#pragma unroll
      for (int ks = 0; ks < 4; ks++) {
        fa[t][ks] = *(lds_bf16x8_ptr)(frd[ks] + stage * 32768 + (wm * 64 + t * 32) * 128);
        fw[t][ks] = *(lds_bf16x8_ptr)(frd[ks] + stage * 32768 + 16384 + (wn * 64 + t * 32) * 128);
      }
#pragma unroll
    for (int ks = 0; ks < 4; ks++)
#pragma unroll
      for (int nt = 0; nt < 2; nt++)
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
          acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[nt][ks], fa[mt][ks], acc[nt][mt], 0, 0, 0);
  }

  // ---- epilogue: lane (token row m = l32, half hh) owns n = 8*ig + 4*hh + 0..3 of each 32x32 tile
#pragma unroll
  for (int mt = 0; mt < 2; mt++) {
    const int m = m0 + wm * 64 + mt * 32 + l32;
    if (m >= p.M) continue;
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        const int n = n0 + wn * 64 + nt * 32 + 8 * ig + 4 * hh;
        const f32x4 b4 = *reinterpret_cast<const f32x4 *>(p.bias + n);
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[e] = acc[nt][mt][4 * ig + e] + b4[e];
          if (p.gelu) o[e] = gelu_erf(o[e]);
        }
        if (p.r) {
          const uint2 r2 = *reinterpret_cast<const uint2 *>(p.r + (size_t)m * p.N + n);
          o[0] += bf16_lo(r2.x); o[1] += bf16_hi(r2.x); o[2] += bf16_lo(r2.y); o[3] += bf16_hi(r2.y);
        }
        uint2 u = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3])};
        *reinterpret_cast<uint2 *>(p.c + (size_t)m * p.N + n) = u;
      }
  }
}

ns_status launch_layernorm(const uint16_t *x, const float *g, const float *b, uint16_t *y, int rows,
                           int dim, float eps, hipStream_t s) {
  dim3 grid((rows + 3) / 4), blk(256);
  switch (dim / 512) {
    case 1: hipLaunchKernelGGL(layernorm_kernel<1>, grid, blk, 0, s, x, g, b, y, rows, eps); break;
    case 2: hipLaunchKernelGGL(layernorm_kernel<2>, grid, blk, 0, s, x, g, b, y, rows, eps); break;
    case 3: hipLaunchKernelGGL(layernorm_kernel<3>, grid, blk, 0, s, x, g, b, y, rows, eps); break;
    case 4: hipLaunchKernelGGL(layernorm_kernel<4>, grid, blk, 0, s, x, g, b, y, rows, eps); break;
    default: return fail(NS_ERR_UNSUPPORTED, "LayerNorm width %d: 512, 1024, 1536 or 2048", dim);
  }
  return check_launch("layernorm_kernel");
}

ns_status launch_gemm(const uint16_t *a, const uint16_t *w, const float *bias, const uint16_t *r,
                      uint16_t *c, int M, int N, int K, bool gelu, hipStream_t s) {
  // NSATTN_GEMM=128 keeps the 128 x 128 kernel for every shape; read once per process
  static const bool only128 = [] { const char *e = getenv("NSATTN_GEMM"); return e && e[0] == '1'; }();
  if (gemm256_supported(M, N, K) && !only128) return launch_gemm256(a, w, bias, r, c, M, N, K, gelu, s);
  if (N % 128 || K % 64) return fail(NS_ERR_UNSUPPORTED, "GEMM needs N %% 128 == 0 and K %% 64 == 0 (N=%d K=%d)", N, K);
  if ((long long)M * K * 2 >= 0x7fffffffLL || (long long)N * K * 2 >= 0x7fffffffLL)
    return fail(NS_ERR_UNSUPPORTED, "GEMM operand beyond 2 GiB");
  GemmParams p{a, w, r, bias, c, M, N, K, gelu ? 1 : 0};
  const long long wgs = (long long)((M + 127) / 128) * (N / 128);
  if (wgs > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "GEMM grid too large");
  hipLaunchKernelGGL(gemm_bf16_kernel, dim3((unsigned)wgs), dim3(256), 65536, s, p);
  return check_launch("gemm_bf16_kernel");
}

struct VitWorkspace {
  size_t ln, qkv, attn, h, hidden, logits, lse, attn_ws, total;
};

VitWorkspace vit_layout(const ns_vit_block_desc &d, const ns_attn_desc &ad) {
  VitWorkspace w;
  const size_t M = (size_t)ad.batch * ad.tokens;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.ln = take(M * d.dim * 2);
  w.qkv = take(M * 3 * d.dim * 2);
  w.attn = take(M * d.dim * 2);
  w.h = take(M * d.dim * 2);
  w.hidden = take(M * d.mlp_dim * 2);
  w.logits = take((size_t)ad.batch * ad.heads * ad.n_global * ad.tokens * 4);
  w.lse = take((size_t)ad.batch * ad.heads * ad.n_global * 4);
  w.attn_ws = off;
  off += align_up(ns_attn_workspace_bytes(&ad), 256);
  w.total = off;
  return w;
}

// The block lays q, k, v out itself: one fused [B,T,3,H,D] projection, attention output [B,T,H,D].
ns_status block_attn_desc(const ns_vit_block_desc *d, ns_attn_desc &ad) {
  if (!d) return fail(NS_ERR_INVALID_ARG, "descriptor is NULL");
  ad = d->attn;
  if (d->dim < 1 || d->mlp_dim < 1) return fail(NS_ERR_INVALID_ARG, "dim and mlp_dim must be positive");
  if (ad.heads < 1 || ad.head_dim < 1 || (long long)ad.heads * ad.head_dim != d->dim)
    return fail(NS_ERR_INVALID_ARG, "heads * head_dim must equal dim");
  if (ad.dtype != NS_BF16) return fail(NS_ERR_UNSUPPORTED, "the block is implemented for bf16 activations");
  if (!(d->ln_eps > 0.f)) return fail(NS_ERR_INVALID_ARG, "ln_eps must be positive");
  if (d->dim % 512 || d->dim > 2048) return fail(NS_ERR_UNSUPPORTED, "dim %d: 512, 1024, 1536 or 2048", d->dim);
  if (d->mlp_dim % 128) return fail(NS_ERR_UNSUPPORTED, "mlp_dim must be a multiple of 128");
  ad.q_stride_t = 3LL * d->dim; ad.q_stride_h = ad.head_dim; ad.q_stride_b = (int64_t)ad.tokens * 3 * d->dim;
  ad.out_stride_t = d->dim; ad.out_stride_h = ad.head_dim; ad.out_stride_b = (int64_t)ad.tokens * d->dim;
  return NS_OK;
}

// idx[i] = r * grid_w + c of the packed position (r << 16 | c): the original patch index of a survivor
__global__ __launch_bounds__(256) void coords_to_index_kernel(const int32_t *coords, int32_t *idx, size_t n, int grid_w) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint32_t pc = (uint32_t)coords[i];
  idx[i] = (int32_t)((pc >> 16) * (uint32_t)grid_w + (pc & 0xffffu));
}

// y[b][j][:] = x[b][G + j][:]: the patch rows of a sequence without its global rows, 16 bytes per
// lane.  grid (ceil(N * vec_per_row / 256), B).
__global__ __launch_bounds__(256) void patch_rows_kernel(const uint4 *x, uint4 *y, int N, int G, int vec_per_row) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x, n = (size_t)N * vec_per_row;
  if (i >= n) return;
  const size_t b = blockIdx.y;
  y[b * n + i] = x[(b * (size_t)(N + G) + G) * vec_per_row + i];
}

// coords[b][j] = (r << 16 | c) of patch j of the full raster grid
// Patch embedding, step 1: the pixels of every patch as one row of a matrix [B*N, Kp] bf16, column
// (c * ps + py) * ps + px (the order of a convolution weight [dim, channels, ps, ps]), columns
// K..Kp-1 zero.  One thread per 8 consecutive columns.
__global__ __launch_bounds__(256) void patch_matrix_kernel(const uint16_t *pixels, uint16_t *a, int channels,
                                                           int grid_h, int grid_w, int ps, int K, int Kp,
                                                           long long total8) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= total8) return;
  const int per_row = Kp / 8;
  const long long row = t / per_row;                 // b * N + patch
  const int col0 = (int)(t - row * per_row) * 8;
  const int N = grid_h * grid_w;
  const int b = (int)(row / N), n = (int)(row - (long long)b * N);
  const int pr = n / grid_w, pc = n - pr * grid_w;
  const long long W = (long long)grid_w * ps, plane = (long long)grid_h * ps * W;
  const uint16_t *img = pixels + (long long)b * channels * plane;
  uint16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; e++) {
    const int col = col0 + e;
    uint16_t x = 0;
    if (col < K) {
      const int c = col / (ps * ps), rem = col - c * ps * ps, py = rem / ps, px = rem - py * ps;
      x = img[c * plane + ((long long)pr * ps + py) * W + (long long)pc * ps + px];
    }
    v[e] = x;
  }
  uint4 u = {(uint32_t)v[0] | ((uint32_t)v[1] << 16), (uint32_t)v[2] | ((uint32_t)v[3] << 16),
             (uint32_t)v[4] | ((uint32_t)v[5] << 16), (uint32_t)v[6] | ((uint32_t)v[7] << 16)};
  *reinterpret_cast<uint4 *>(a + row * Kp + col0) = u;
}

// rows [rows, K] -> [rows, Kp], new columns zero (the projection weight, when K is no multiple of 64)
__global__ __launch_bounds__(256) void pad_columns_kernel(const uint16_t *w, uint16_t *wp, int rows, int K, int Kp) {
  const long long t = (long long)blockIdx.x * 256 + threadIdx.x;
  if (t >= (long long)rows * Kp) return;
  const int r = (int)(t / Kp), c = (int)(t - (long long)r * Kp);
  wp[t] = c < K ? w[(long long)r * K + c] : (uint16_t)0;
}

// x[b, 0, :] = cls_token + pos_embed[0, :]
__global__ __launch_bounds__(256) void cls_rows_kernel(const uint16_t *cls, const uint16_t *pos, uint16_t *x,
                                                       int dim, long long image_stride) {
  const int d = blockIdx.x * 256 + threadIdx.x;
  if (d >= dim) return;
  const float v = bf16_lo((uint32_t)cls[d]) + bf16_lo((uint32_t)pos[d]);
  x[(long long)blockIdx.y * image_stride + d] = (uint16_t)(pack_bf16(v, 0.f) & 0xffffu);
}

__global__ __launch_bounds__(256) void raster_coords_kernel(int32_t *coords, int n, int grid_w) {
  const int j = blockIdx.x * 256 + threadIdx.x;
  if (j < n) coords[(size_t)blockIdx.y * n + j] = ((j / grid_w) << 16) | (j % grid_w);
}

struct StackWorkspace {
  size_t xa, xb, scores, kept, coords_in, coords_out, block_ws, total;
};

StackWorkspace stack_layout(const ns_vit_desc &d, size_t block_ws_bytes) {
  StackWorkspace w;
  const ns_attn_desc &a = d.block.attn;
  const size_t xbytes = (size_t)a.batch * a.tokens * d.block.dim * 2, N = (size_t)a.tokens - a.n_global;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  w.xa = take(xbytes);
  w.xb = take(xbytes);
  w.scores = take((size_t)a.batch * N * 4);
  w.kept = take((size_t)a.batch * N * 4);
  w.coords_in = take((size_t)a.batch * N * 4);
  w.coords_out = take((size_t)a.batch * N * 4);
  w.block_ws = off;
  off += align_up(block_ws_bytes, 256);
  w.total = off;
  return w;
}

ns_status check_stack(const ns_vit_desc *d, bool &prune) {
  if (!d) return fail(NS_ERR_INVALID_ARG, "descriptor is NULL");
  if (d->layers < 1) return fail(NS_ERR_INVALID_ARG, "layers must be positive");
  if (d->block.attn.coords) return fail(NS_ERR_INVALID_ARG, "the stack starts from the full grid: attn.coords must be NULL");
  prune = d->prune_after > 0 && d->keep_k > 0;
  if (d->prune_after < 0 || d->prune_after > d->layers) return fail(NS_ERR_INVALID_ARG, "prune_after out of range");
  if (prune && d->keep_k > d->block.attn.tokens - d->block.attn.n_global)
    return fail(NS_ERR_INVALID_ARG, "keep_k exceeds the number of patches");
  if (d->keep_k < 0) return fail(NS_ERR_INVALID_ARG, "keep_k must not be negative");
  return NS_OK;
}

// Stage lists: block numbers strictly ascending in 1..layers, keep counts positive, at most the
// number of patches and never growing.
ns_status check_stages(const ns_vit_desc *d, int n_stages, const int32_t *after, const int32_t *keep) {
  if (!d) return fail(NS_ERR_INVALID_ARG, "descriptor is NULL");
  if (d->layers < 1) return fail(NS_ERR_INVALID_ARG, "layers must be positive");
  if (d->block.attn.coords) return fail(NS_ERR_INVALID_ARG, "the stack starts from the full grid: attn.coords must be NULL");
  if (n_stages < 0 || n_stages > d->layers) return fail(NS_ERR_INVALID_ARG, "n_stages out of range");
  if (n_stages > 0 && (!after || !keep)) return fail(NS_ERR_INVALID_ARG, "stage arrays are NULL");
  const int N = d->block.attn.tokens - d->block.attn.n_global;
  for (int i = 0; i < n_stages; i++) {
    if (after[i] < 1 || after[i] > d->layers || (i > 0 && after[i] <= after[i - 1]))
      return fail(NS_ERR_INVALID_ARG, "stage_after must be strictly ascending in 1..layers");
    if (keep[i] < 1 || keep[i] > (i > 0 ? keep[i - 1] : N))
      return fail(NS_ERR_INVALID_ARG, "stage_keep must be positive, at most the number of patches, and not grow");
  }
  return NS_OK;
}

}  // namespace
}  // namespace ns

using namespace ns;

static ns_status block_forward_impl(const ns_vit_block_desc *desc, const ns_vit_block_weights *w,
                                    const void *x_in, void *x_out, float *scores_out, void *workspace,
                                    size_t workspace_bytes, void *stream, bool reuse_lists);

extern "C" {

size_t vit_block_workspace_bytes(const ns_vit_block_desc *desc) {
  ns_attn_desc ad;
  if (block_attn_desc(desc, ad) != NS_OK) return 0;
  if (ns_attn_workspace_bytes(&ad) == 0) return 0;   // invalid attention descriptor
  return vit_layout(*desc, ad).total;
}

ns_status vit_block_forward(const ns_vit_block_desc *desc, const ns_vit_block_weights *w,
                            const void *x_in, void *x_out, float *scores_out, void *workspace,
                            size_t workspace_bytes, void *stream) {
  return block_forward_impl(desc, w, x_in, x_out, scores_out, workspace, workspace_bytes, stream, false);
}

}  // extern "C"

// reuse_lists: see attn_forward_impl
static ns_status block_forward_impl(const ns_vit_block_desc *desc, const ns_vit_block_weights *w,
                                    const void *x_in, void *x_out, float *scores_out, void *workspace,
                                    size_t workspace_bytes, void *stream, bool reuse_lists) {
  ns_attn_desc ad;
  ns_status st = block_attn_desc(desc, ad);
  if (st != NS_OK) return st;
  st = attn_validate(&ad);
  if (st != NS_OK) return st;
  if (!w || !x_in || !x_out) return fail(NS_ERR_INVALID_ARG, "weights, x_in and x_out must not be NULL");
  if (!w->ln1_g || !w->ln1_b || !w->w_qkv || !w->b_qkv || !w->w_proj || !w->b_proj || !w->ln2_g ||
      !w->ln2_b || !w->w_fc1 || !w->b_fc1 || !w->w_fc2 || !w->b_fc2)
    return fail(NS_ERR_INVALID_ARG, "a weight pointer is NULL");
  if (x_in == x_out) return fail(NS_ERR_INVALID_ARG, "x_out must not alias x_in");
  if (reinterpret_cast<uintptr_t>(x_in) % 16 || reinterpret_cast<uintptr_t>(x_out) % 16)
    return fail(NS_ERR_INVALID_ARG, "x_in and x_out must be 16-byte aligned");
  const VitWorkspace L = vit_layout(*desc, ad);
  if (!workspace) return fail(NS_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", L.total);
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(NS_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < L.total)
    return fail(NS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);

  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  uint16_t *ln = reinterpret_cast<uint16_t *>(ws + L.ln), *qkv = reinterpret_cast<uint16_t *>(ws + L.qkv);
  uint16_t *att = reinterpret_cast<uint16_t *>(ws + L.attn), *h = reinterpret_cast<uint16_t *>(ws + L.h);
  uint16_t *hid = reinterpret_cast<uint16_t *>(ws + L.hidden);
  float *logits = reinterpret_cast<float *>(ws + L.logits), *lse = reinterpret_cast<float *>(ws + L.lse);
  const uint16_t *x = static_cast<const uint16_t *>(x_in);
  uint16_t *y = static_cast<uint16_t *>(x_out);
  const int M = ad.batch * ad.tokens, dim = desc->dim, mlp = desc->mlp_dim;

  st = launch_layernorm(x, w->ln1_g, w->ln1_b, ln, M, dim, desc->ln_eps, s);
  if (st != NS_OK) return st;
  st = launch_gemm(ln, static_cast<const uint16_t *>(w->w_qkv), w->b_qkv, nullptr, qkv, M, 3 * dim, dim, false, s);
  if (st != NS_OK) return st;
  st = attn_forward_impl(&ad, qkv, qkv + dim, qkv + 2 * dim, att, scores_out ? logits : nullptr,
                         scores_out ? lse : nullptr, scores_out, ws + L.attn_ws, L.total - L.attn_ws, s,
                         reuse_lists);
  if (st != NS_OK) return st;
  st = launch_gemm(att, static_cast<const uint16_t *>(w->w_proj), w->b_proj, x, h, M, dim, dim, false, s);
  if (st != NS_OK) return st;
  st = launch_layernorm(h, w->ln2_g, w->ln2_b, ln, M, dim, desc->ln_eps, s);
  if (st != NS_OK) return st;
  st = launch_gemm(ln, static_cast<const uint16_t *>(w->w_fc1), w->b_fc1, nullptr, hid, M, mlp, dim, true, s);
  if (st != NS_OK) return st;
  return launch_gemm(hid, static_cast<const uint16_t *>(w->w_fc2), w->b_fc2, h, y, M, dim, mlp, false, s);
}

// Workspace of one block of the stack: the larger of what a block on the full grid and a block on
// the pruned sequence need (the latter also holds per-block token lists and counts, and with a
// keep count within a few tokens of the grid size that is more than the full grid's).
static size_t stack_block_workspace_bytes(const ns_vit_desc &d, bool prune) {
  size_t bw = vit_block_workspace_bytes(&d.block);
  if (bw == 0 || !prune) return bw;
  ns_vit_block_desc pd = d.block;
  pd.attn.tokens = d.block.attn.n_global + d.keep_k;
  // (only "not NULL" matters for the size; the pointer is never dereferenced on the host)
  pd.attn.coords = reinterpret_cast<const int32_t *>(static_cast<uintptr_t>(256));
  const size_t pw = vit_block_workspace_bytes(&pd);
  if (pw == 0) return 0;
  return bw > pw ? bw : pw;
}

extern "C" {

size_t vit_workspace_bytes(const ns_vit_desc *desc) {
  bool prune;
  if (check_stack(desc, prune) != NS_OK) return 0;
  const size_t bw = stack_block_workspace_bytes(*desc, prune);
  if (bw == 0) return 0;
  return stack_layout(*desc, bw).total;
}

static ns_status check_embed(int32_t batch, int32_t channels, int32_t grid_h, int32_t grid_w, int32_t patch,
                             int32_t dim) {
  if (batch < 1 || channels < 1 || grid_h < 1 || grid_w < 1 || patch < 1)
    return fail(NS_ERR_INVALID_ARG, "batch, channels, grid and patch must be positive");
  if (dim < 128 || dim % 128) return fail(NS_ERR_UNSUPPORTED, "dim %d: a positive multiple of 128", dim);
  const long long K = (long long)channels * patch * patch, N = (long long)grid_h * grid_w;
  if (K > 65536 || N * align_up((size_t)K, 64) * 2 >= 0x7fffffffLL)
    return fail(NS_ERR_UNSUPPORTED, "patch matrix of one image beyond 2 GiB");
  if ((long long)batch * N >= 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "too many patches");
  return NS_OK;
}

size_t vit_embed_workspace_bytes(int32_t batch, int32_t channels, int32_t grid_h, int32_t grid_w, int32_t patch,
                                 int32_t dim) {
  if (check_embed(batch, channels, grid_h, grid_w, patch, dim) != NS_OK) return 0;
  const size_t K = (size_t)channels * patch * patch, Kp = align_up(K, 64);
  return align_up((size_t)batch * grid_h * grid_w * Kp * 2, 256) + align_up((size_t)dim * Kp * 2, 256);
}

ns_status vit_embed(int32_t batch, int32_t channels, int32_t grid_h, int32_t grid_w, int32_t patch, int32_t dim,
                    const void *pixels, const void *w_patch, const float *b_patch, const void *cls_token,
                    const void *pos_embed, void *x_out, void *workspace, size_t workspace_bytes, void *stream) {
  ns_status st = check_embed(batch, channels, grid_h, grid_w, patch, dim);
  if (st != NS_OK) return st;
  if (!pixels || !w_patch || !b_patch || !cls_token || !pos_embed || !x_out)
    return fail(NS_ERR_INVALID_ARG, "pixels, weights, cls_token, pos_embed and x_out must not be NULL");
  const uintptr_t bits = reinterpret_cast<uintptr_t>(w_patch) | reinterpret_cast<uintptr_t>(b_patch) |
                         reinterpret_cast<uintptr_t>(pos_embed) | reinterpret_cast<uintptr_t>(x_out);
  if (bits % 16 || reinterpret_cast<uintptr_t>(pixels) % 2 || reinterpret_cast<uintptr_t>(cls_token) % 2)
    return fail(NS_ERR_INVALID_ARG, "w_patch, b_patch, pos_embed and x_out must be 16-byte aligned");
  const size_t need = vit_embed_workspace_bytes(batch, channels, grid_h, grid_w, patch, dim);
  if (!workspace) return fail(NS_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", need);
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(NS_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < need) return fail(NS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, need);

  hipStream_t s = static_cast<hipStream_t>(stream);
  const int N = grid_h * grid_w, K = channels * patch * patch, Kp = (int)align_up((size_t)K, 64);
  uint16_t *a = static_cast<uint16_t *>(workspace);
  uint16_t *wp = reinterpret_cast<uint16_t *>(static_cast<unsigned char *>(workspace) +
                                              align_up((size_t)batch * N * Kp * 2, 256));
  const uint16_t *w = static_cast<const uint16_t *>(w_patch);
  const long long total8 = (long long)batch * N * (Kp / 8);
  hipLaunchKernelGGL(patch_matrix_kernel, dim3((unsigned)((total8 + 255) / 256)), dim3(256), 0, s,
                     static_cast<const uint16_t *>(pixels), a, channels, grid_h, grid_w, patch, K, Kp, total8);
  st = check_launch("patch_matrix_kernel");
  if (st != NS_OK) return st;
  if (Kp != K) {
    hipLaunchKernelGGL(pad_columns_kernel, dim3((unsigned)(((long long)dim * Kp + 255) / 256)), dim3(256), 0, s, w, wp,
                       dim, K, Kp);
    st = check_launch("pad_columns_kernel");
    if (st != NS_OK) return st;
    w = wp;
  }
  const uint16_t *pos = static_cast<const uint16_t *>(pos_embed);
  uint16_t *x = static_cast<uint16_t *>(x_out);
  const long long image_stride = (long long)(1 + N) * dim;
  for (int b = 0; b < batch; b++) {
    // rows 1..N of image b: projection + bias, the position embeddings ride in as the residual
    st = launch_gemm(a + (size_t)b * N * Kp, w, b_patch, pos + dim, x + b * image_stride + dim, N, dim, Kp, false, s);
    if (st != NS_OK) return st;
  }
  hipLaunchKernelGGL(cls_rows_kernel, dim3((dim + 255) / 256, batch), dim3(256), 0, s,
                     static_cast<const uint16_t *>(cls_token), pos, x, dim, image_stride);
  return check_launch("cls_rows_kernel");
}

ns_status linear_forward(int32_t M, int32_t N, int32_t K, const void *x, const void *w, const float *bias,
                         const void *residual, int32_t gelu, void *y, void *stream) {
  if (M <= 0 || N <= 0 || K <= 0) return fail(NS_ERR_INVALID_ARG, "M, N, K must be positive");
  if (!x || !w || !bias || !y) return fail(NS_ERR_INVALID_ARG, "x, w, bias and y must not be NULL");
  const uintptr_t bits = reinterpret_cast<uintptr_t>(x) | reinterpret_cast<uintptr_t>(w) |
                         reinterpret_cast<uintptr_t>(bias) | reinterpret_cast<uintptr_t>(residual) |
                         reinterpret_cast<uintptr_t>(y);
  if (bits % 16) return fail(NS_ERR_INVALID_ARG, "pointers must be 16-byte aligned");
  if (y == x || y == w || y == residual) return fail(NS_ERR_INVALID_ARG, "y must not alias an input");
  return launch_gemm(static_cast<const uint16_t *>(x), static_cast<const uint16_t *>(w), bias,
                     static_cast<const uint16_t *>(residual), static_cast<uint16_t *>(y), M, N, K, gelu != 0,
                     static_cast<hipStream_t>(stream));
}

ns_status vit_forward(const ns_vit_desc *desc, const ns_vit_block_weights *weights, const void *x_in,
                      void *x_out, int32_t *kept_idx, void *workspace, size_t workspace_bytes,
                      void *stream) {
  return vit_forward_features(desc, weights, x_in, x_out, kept_idx, 0, nullptr, nullptr, workspace,
                              workspace_bytes, stream);
}

// The stack with a list of pruning stages (HOST arrays, validated by the caller): shared by the
// entry points below.  `d` carries the first stage in prune_after / keep_k (or none), which is what
// the workspace is sized for.
static ns_status stack_run(const ns_vit_desc &d, int n_stages, const int32_t *after, const int32_t *keep,
                           const ns_vit_block_weights *weights, const void *x_in, void *x_out, int32_t *kept_idx,
                           int32_t n_taps, const int32_t *tap_layers, void *const *tap_out, void *workspace,
                           size_t workspace_bytes, void *stream) {
  const bool prune = n_stages > 0;
  ns_status st;
  if (n_taps < 0 || (n_taps > 0 && (!tap_layers || !tap_out)))
    return fail(NS_ERR_INVALID_ARG, "n_taps must be >= 0 and the tap arrays given with it");
  for (int i = 0; i < n_taps; i++) {
    if (tap_layers[i] < 1 || tap_layers[i] > d.layers || (i > 0 && tap_layers[i] <= tap_layers[i - 1]))
      return fail(NS_ERR_INVALID_ARG, "tap_layers must be ascending in 1..layers");
    if (prune && tap_layers[i] > after[0])
      return fail(NS_ERR_INVALID_ARG, "a feature map after the pruning stage has no grid structure left");
    if (!tap_out[i] || reinterpret_cast<uintptr_t>(tap_out[i]) % 16)
      return fail(NS_ERR_INVALID_ARG, "tap_out[%d] is NULL or misaligned", i);
  }
  const size_t bw = stack_block_workspace_bytes(d, prune);
  if (bw == 0) {                      // the block's own validation says why: pass its status on
    ns_attn_desc ad;
    st = block_attn_desc(&d.block, ad);
    if (st == NS_OK) st = attn_validate(&ad);
    return st != NS_OK ? st : fail(NS_ERR_INVALID_ARG, "invalid block descriptor");
  }
  if (!weights || !x_in || !x_out) return fail(NS_ERR_INVALID_ARG, "weights, x_in and x_out must not be NULL");
  const StackWorkspace L = stack_layout(d, bw);
  if (!workspace) return fail(NS_ERR_WORKSPACE, "workspace is NULL, %zu bytes needed", L.total);
  if (reinterpret_cast<uintptr_t>(workspace) % 256) return fail(NS_ERR_WORKSPACE, "workspace must be 256-byte aligned");
  if (workspace_bytes < L.total) return fail(NS_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  void *buf[2] = {ws + L.xa, ws + L.xb};
  float *scores = reinterpret_cast<float *>(ws + L.scores);
  int32_t *kept_ws = reinterpret_cast<int32_t *>(ws + L.kept);
  // the survivors' grid positions: read from one list, written to the other, stage by stage
  int32_t *cbuf[2] = {reinterpret_cast<int32_t *>(ws + L.coords_in), reinterpret_cast<int32_t *>(ws + L.coords_out)};
  int cflip = 0;

  ns_vit_block_desc bd = d.block;
  const ns_attn_desc full = d.block.attn;
  const int N = full.tokens - full.n_global;
  int n_cur = N;              // patches in the sequence
  const void *cur = x_in;
  int flip = 0;
  bool lists_built = false;   // block lists stay valid from block to block until the sequence changes
  int tap = 0, stage = 0;
  for (int l = 0; l < d.layers; l++) {
    const bool last = l + 1 == d.layers, scoring = stage < n_stages && l + 1 == after[stage];
    // the last block writes x_out directly unless a pruning stage still follows it
    void *dst = (last && !scoring) ? x_out : buf[flip];
    st = block_forward_impl(&bd, &weights[l], cur, dst, scoring ? scores : nullptr, ws + L.block_ws, bw, s,
                            lists_built);
    if (st != NS_OK) return st;
    lists_built = true;
    cur = dst;
    flip ^= 1;
    if (tap < n_taps && tap_layers[tap] == l + 1) {
      const int vec = bd.dim * 2 / 16;
      dim3 grid((unsigned)(((size_t)N * vec + 255) / 256), full.batch);
      hipLaunchKernelGGL(patch_rows_kernel, grid, dim3(256), 0, s, static_cast<const uint4 *>(cur),
                         static_cast<uint4 *>(tap_out[tap]), N, full.n_global, vec);
      st = check_launch("patch_rows_kernel");
      if (st != NS_OK) return st;
      tap++;
    }
    if (scoring) {
      int32_t *cin = cbuf[cflip], *cout = cbuf[cflip ^ 1];
      if (stage == 0) {
        dim3 grid((N + 255) / 256, full.batch);
        hipLaunchKernelGGL(raster_coords_kernel, grid, dim3(256), 0, s, cin, N, full.grid_w);
        st = check_launch("raster_coords_kernel");
        if (st != NS_OK) return st;
      }
      const int k = keep[stage];
      // the first stage's indices are the original patch indices: with one stage they go straight to the caller
      int32_t *kept = (n_stages == 1 && kept_idx) ? kept_idx : kept_ws;
      void *y = last ? x_out : buf[flip];
      st = topk_filter_global(full.batch, n_cur, k, full.n_global, scores, cur, bd.dim, NS_BF16, cin, kept,
                              y, cout, ws + L.block_ws, bw, s);   // the block's workspace is idle here
      if (st != NS_OK) return st;
      cur = y;
      flip ^= 1;
      cflip ^= 1;
      n_cur = k;
      bd.attn.tokens = full.n_global + k;
      bd.attn.coords = cout;
      lists_built = false;
      stage++;
      if (stage == n_stages && n_stages > 1 && kept_idx) {
        // later stages select among survivors: the original indices come from the positions
        const size_t n = (size_t)full.batch * k;
        hipLaunchKernelGGL(coords_to_index_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, cout, kept_idx, n,
                           full.grid_w);
        st = check_launch("coords_to_index_kernel");
        if (st != NS_OK) return st;
      }
    }
  }
  return NS_OK;
}

ns_status vit_forward_features(const ns_vit_desc *desc, const ns_vit_block_weights *weights, const void *x_in,
                               void *x_out, int32_t *kept_idx, int32_t n_taps, const int32_t *tap_layers,
                               void *const *tap_out, void *workspace, size_t workspace_bytes, void *stream) {
  bool prune;
  ns_status st = check_stack(desc, prune);
  if (st != NS_OK) return st;
  const int32_t after = desc->prune_after, keep = desc->keep_k;
  return stack_run(*desc, prune ? 1 : 0, &after, &keep, weights, x_in, x_out, kept_idx, n_taps, tap_layers, tap_out,
                   workspace, workspace_bytes, stream);
}

size_t vit_stages_workspace_bytes(const ns_vit_desc *desc, int32_t n_stages, const int32_t *stage_after,
                                  const int32_t *stage_keep) {
  if (check_stages(desc, n_stages, stage_after, stage_keep) != NS_OK) return 0;
  ns_vit_desc d = *desc;
  d.prune_after = n_stages ? stage_after[0] : 0;
  d.keep_k = n_stages ? stage_keep[0] : 0;
  return vit_workspace_bytes(&d);
}

ns_status vit_forward_stages(const ns_vit_desc *desc, int32_t n_stages, const int32_t *stage_after,
                             const int32_t *stage_keep, const ns_vit_block_weights *weights, const void *x_in,
                             void *x_out, int32_t *kept_idx, void *workspace, size_t workspace_bytes, void *stream) {
  const ns_status st = check_stages(desc, n_stages, stage_after, stage_keep);
  if (st != NS_OK) return st;
  ns_vit_desc d = *desc;
  d.prune_after = n_stages ? stage_after[0] : 0;
  d.keep_k = n_stages ? stage_keep[0] : 0;
  return stack_run(d, n_stages, stage_after, stage_keep, weights, x_in, x_out, kept_idx, 0, nullptr, nullptr, workspace,
                   workspace_bytes, stream);
}

}  // extern "C"
