// Internal helpers shared by the HIP translation units of libnsattn.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/nsattn.h"

namespace ns {

// ---- error reporting -------------------------------------------------------
ns_status fail(ns_status code, const char *fmt, ...);
ns_status check_launch(const char *what);   // hipGetLastError -> NS_ERR_HIP

// ---- bf16 <-> fp32 on the device ------------------------------------------
typedef __bf16 bf16_t;
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// round-to-nearest-even pack of two floats into two bf16 (v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  f32x2 v = {lo, hi};
  bf16x2 r = __builtin_convertvector(v, bf16x2);
  return __builtin_bit_cast(uint32_t, r);
}

constexpr float kLog2e = 1.4426950408889634f;

// GELU with the Gaussian error function, 0.5 x (1 + erf(x / sqrt 2)), written so that the
// cancellation for negative x never happens: with z = |x| / sqrt 2 and E = erfc(z),
//   gelu(x) = max(x, 0) - |x| (E / 2).
// erfc(z) = t (a1 + t (a2 + t (a3 + t (a4 + t a5)))) exp(-z^2), t = 1 / (1 + p z), is the rational
// approximation 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7, i.e. at the level of
// fp32 rounding and far below the bf16 rounding of the result).  The factors 1/2 and 1/sqrt 2 are
// folded into the constants: 13 vector instructions per value.
__device__ __forceinline__ float gelu_erf(float x) {
  const float ax = __builtin_fabsf(x);
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f * 0.70710678118654752f, ax, 1.f));
  float q = __builtin_fmaf(0.5f * 1.061405429f, t, 0.5f * -1.453152027f);
  q = __builtin_fmaf(q, t, 0.5f * 1.421413741f);
  q = __builtin_fmaf(q, t, 0.5f * -0.284496736f);
  q = __builtin_fmaf(q, t, 0.5f * 0.254829592f);
  const float e = __builtin_amdgcn_exp2f((x * x) * (-0.5f * 1.4426950408889634f));
  const float E = q * t * e;
  return __builtin_fmaf(-ax, E, __builtin_fmaxf(x, 0.f));
}
// The same for eight values, stage by stage, so that the eight dependency chains (two of their
// links are transcendental instructions with a long result latency) are interleaved: a wave that
// has its SIMD to itself otherwise waits out every link.  The empty asm statements between the
// stages keep the compiler from putting the chains back one after the other.
__device__ __forceinline__ void stage8(float (&a)[8]) {
  asm volatile("" : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7]));
}
__device__ __forceinline__ void gelu_erf8(float (&o)[8]) {
  float t[8], e[8], q[8], r[8];
#pragma unroll
  for (int i = 0; i < 8; i++) t[i] = __builtin_fmaf(0.3275911f * 0.70710678118654752f, __builtin_fabsf(o[i]), 1.f);
  stage8(t);
#pragma unroll
  for (int i = 0; i < 8; i++) r[i] = __builtin_fmaxf(o[i], 0.f);
  stage8(r);
#pragma unroll
  for (int i = 0; i < 8; i++) t[i] = __builtin_amdgcn_rcpf(t[i]);
  stage8(t);
#pragma unroll
  for (int i = 0; i < 8; i++) e[i] = (o[i] * o[i]) * (-0.5f * 1.4426950408889634f);
  stage8(e);
#pragma unroll
  for (int i = 0; i < 8; i++) e[i] = __builtin_amdgcn_exp2f(e[i]);
  stage8(e);
#pragma unroll
  for (int i = 0; i < 8; i++) q[i] = __builtin_fmaf(0.5f * 1.061405429f, t[i], 0.5f * -1.453152027f);
  stage8(q);
#pragma unroll
  for (int i = 0; i < 8; i++) q[i] = __builtin_fmaf(q[i], t[i], 0.5f * 1.421413741f);
  stage8(q);
#pragma unroll
  for (int i = 0; i < 8; i++) q[i] = __builtin_fmaf(q[i], t[i], 0.5f * -0.284496736f);
  stage8(q);
#pragma unroll
  for (int i = 0; i < 8; i++) q[i] = __builtin_fmaf(q[i], t[i], 0.5f * 0.254829592f);
  stage8(q);
#pragma unroll
  for (int i = 0; i < 8; i++) e[i] *= q[i] * t[i];
  stage8(e);
#pragma unroll
  for (int i = 0; i < 8; i++) o[i] = __builtin_fmaf(-__builtin_fabsf(o[i]), e[i], r[i]);
  stage8(o);
}
constexpr float kLn2 = 0.6931471805599453f;

// ---- geometry of the block neighbourhood ----------------------------------
// Everything a kernel needs to turn (block, slot) into a token index.  With lists == nullptr
// the sequence is the full raster grid and the mapping is analytic; otherwise (pruned
// sequence) lists[b][blk][slot] holds the token index and counts[b][blk] the fill.
struct BlockGeom {
  int grid_h, grid_w, block, nbh, nbw, n_global, tokens;
  int cap;                 // block*block: slots per block in `lists`
  const int32_t *lists;    // [B, nbh*nbw, cap] or nullptr
  const int32_t *counts;   // [B, nbh*nbw]      or nullptr
};

__device__ __forceinline__ int block_count(const BlockGeom &g, int b, int R, int C) {
  if (g.counts) return g.counts[(size_t)b * g.nbh * g.nbw + R * g.nbw + C];
  int bh = min(g.block, g.grid_h - R * g.block);
  int bw = min(g.block, g.grid_w - C * g.block);
  return bh * bw;
}

__device__ __forceinline__ int block_token(const BlockGeom &g, int b, int R, int C, int slot) {
  if (g.lists) return g.lists[((size_t)b * g.nbh * g.nbw + R * g.nbw + C) * g.cap + slot];
  int bw = min(g.block, g.grid_w - C * g.block);
  int r = R * g.block + slot / bw;
  int c = C * g.block + slot % bw;
  return g.n_global + r * g.grid_w + c;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- device helpers shared by the MFMA kernels ------------------------------
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// A value the compiler can no longer trace back: what is computed from it stays where it is written
// instead of being hoisted out of a loop into registers that live for the whole kernel.
__device__ __forceinline__ int opaque(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// max / sum of a value over the two half-waves (lane l and lane l ^ 32); both lanes get it
__device__ __forceinline__ float half_swap_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// 16 bytes per lane, global -> LDS, no registers: LDS address = lds + 16 * lane.  Issued as asm
// so that the compiler does not guard later LDS reads with a full vmcnt(0) wait (it cannot tell
// one tile's transfer from the next tile's, which is still in flight); the kernels order and
// count their memory requests themselves (wait_vm).
__device__ __forceinline__ void dma16(const char *base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds), "v"(voff), "s"(base) : "memory", "m0");
}
// 4 / 8 bytes per lane to global memory, issued from asm so that each is exactly one request
__device__ __forceinline__ void store4(void *ptr, float v) {
  asm volatile("global_store_dword %0, %1, off" :: "v"(ptr), "v"(v) : "memory");
}
__device__ __forceinline__ void store8(void *ptr, u32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off" :: "v"(ptr), "v"(v) : "memory");
}
// at most N vector memory requests of this wave still in flight (they complete in issue order)
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// ---- host helpers -------------------------------------------------------------
// Compute units of the current device (256 if the query fails).  Thread-safe; looked up once.
int device_cu_count();
// hipFuncSetAttribute(MaxDynamicSharedMemorySize) for a kernel that wants more than 64 KB of LDS;
// every kernel is set up once per process (thread-safe).  `slot` tells the kernels of a file apart.
ns_status reserve_lds_once(const void *kernel, int bytes);


// ---- launchers implemented in the individual .hip files --------------------
struct AttnArgs {
  ns_attn_desc d;
  const void *q, *k, *v;
  void *out;
  BlockGeom geom;
  hipStream_t stream;
  int kernel;            // the patch-query kernel chosen for this call (ns_api.hip: PatchKernel)
};

// ns_attn_forward with one more knob: reuse_lists = the per-block token lists that an earlier call
// with the same descriptor, coords contents and workspace left in the workspace are still valid
// (a stack of blocks after its pruning stage), so they are not rebuilt.  scores != NULL: also the
// importance scores [B, T-G] (needs cls_logits), merged and scored in one launch.
ns_status attn_forward_impl(const ns_attn_desc *desc, const void *q, const void *k, const void *v, void *out,
                            float *cls_logits, float *cls_lse, float *scores, void *workspace,
                            size_t workspace_bytes, void *stream, bool reuse_lists);

// the descriptor checks of ns_attn_forward alone (status and message as that call would give)
ns_status attn_validate(const ns_attn_desc *desc);

// cls_scores behind its validation: shared by the entry point that takes a workspace and the one
// that brings its own scratch memory
ns_status cls_scores_impl(const ns_attn_desc *desc, const void *q, const void *k, float *scores,
                          void *workspace, size_t workspace_bytes, void *stream);

ns_status launch_block_lists(const ns_attn_desc &d, int32_t *lists, int32_t *counts, hipStream_t s);
ns_status launch_grid_lists(const ns_attn_desc &d, int32_t *lists, int32_t *counts, hipStream_t s);
ns_status launch_attn_generic(const AttnArgs &a);
bool mfma_attn_supported(const ns_attn_desc &d);
ns_status launch_attn_mfma(const AttnArgs &a);
bool persist_attn_supported(const ns_attn_desc &d);
ns_status launch_attn_persist(const AttnArgs &a);
bool sweep_attn_supported(const ns_attn_desc &d);    // 8x8 blocks: key tiles shared along a row of blocks
// cls_partials != NULL: the kernel also computes the global query's row, [B,H,4*nbh,66] partial records
// (sweep_cls_chunks of them per head-image) and, with cls_logits, its raw logits [B,H,T]
ns_status launch_attn_sweep(const AttnArgs &a, float *cls_logits, float *cls_partials);
inline int sweep_cls_chunks(const ns_attn_desc &d) { return 4 * ((d.grid_h + 7) / 8); }
bool block16_attn_supported(const ns_attn_desc &d);  // 16x16 blocks: key tiles shared by a block's four query tiles
ns_status launch_attn_block16(const AttnArgs &a);
bool ragged_attn_supported(const ns_attn_desc &d);   // bf16, head_dim 64: anything given per-block token lists
ns_status launch_attn_ragged(const AttnArgs &a);

// global-query (CLS) row: per-chunk partials, then a combine.
constexpr int kClsChunk = 512;                      // keys per workgroup of the row kernel
inline int cls_num_chunks(int tokens) { return (tokens + kClsChunk - 1) / kClsChunk; }
// partial record per (b, h, chunk): m, l, o[64]
constexpr int kClsPartialFloats = 2 + 64;
ns_status launch_cls_row(const ns_attn_desc &d, const void *q, const void *k, const void *v,
                         float *logits /* [B,H,T] */, float *partials, bool with_v, hipStream_t s);
ns_status launch_cls_combine(const ns_attn_desc &d, const float *partials, void *out, float *lse,
                             bool with_v, hipStream_t s, int nchunks = 0 /* 0: cls_num_chunks(tokens) */);
// lse given directly, or (lse == nullptr) recomputed from the row kernel's partials
// launch_cls_combine and the scoring of all patches in one launch (lse may be NULL)
ns_status launch_cls_combine_scores(const ns_attn_desc &d, const float *partials, void *out, float *lse,
                                    const float *logits, float *scores, hipStream_t s, int nchunks = 0);
ns_status launch_cls_scores(int B, int H, int T, int G, const float *logits, const float *lse,
                            const float *partials, int nchunks, float *scores, hipStream_t s);

// linear map with fused epilogue, 256 x 256 workgroup tiles (ns_gemm256.hip)
bool gemm256_supported(int M, int N, int K);
ns_status launch_gemm256(const uint16_t *a, const uint16_t *w, const float *bias, const uint16_t *r,
                         uint16_t *c, int M, int N, int K, bool gelu, hipStream_t s);

// ws: topk_select_workspace_bytes(B, N) bytes, 16-byte aligned (nothing for short score rows)
size_t topk_select_workspace_bytes(int B, int N);
ns_status launch_topk_select(int B, int N, int k, const float *scores, const int32_t *coords_in,
                             int32_t *kept, int32_t *coords_out, void *ws, hipStream_t s);
ns_status launch_gather_rows(int B, int N, int k, int G, size_t row_bytes, const void *x,
                             const int32_t *kept, void *y, hipStream_t s);

}  // namespace ns
