// The global (CLS) query's attention row and the importance scores derived from it.
//
// Paper, "Memory-Efficiency Optimization": the global token attends to every token.
// Paper, "Time-Efficiency Optimization": a per-token importance score is read off the
// global token's attention weights; here: softmax weight of CLS on each patch key, averaged
// over heads.
//
// One query against T keys is a bandwidth problem, so the row is cut into chunks of 512
// keys: cls_row_kernel streams K (and V) once, writes the raw logits and one softmax
// partial (max, sum, weighted V sum) per chunk; cls_combine_kernel merges the partials in
// chunk order; cls_scores_kernel turns logits + log-sum-exp into head-averaged weights.
#include "ns_common.h"

namespace ns {

namespace {

template <typename T> struct Row8;   // 8 consecutive elements of a row as floats
template <> struct Row8<float> {
  template <bool STREAM = false>
  __device__ static void load(const float *p, float (&x)[8]) {
    f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; e++) { x[e] = a[e]; x[4 + e] = b[e]; }
  }
};
template <> struct Row8<uint16_t> {
  // STREAM: non-temporal load.  Measured: 10 % faster where K and V are both streamed (51 against
  // 57 us on a 256 x 256 grid), 15 % slower where only K is read, so only the former uses it.
  template <bool STREAM = false>
  __device__ static void load(const uint16_t *p, float (&x)[8]) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 *pv = reinterpret_cast<const u32x4 *>(p);
    const u32x4 u = STREAM ? __builtin_nontemporal_load(pv) : *pv;
    x[0] = bf16_lo(u[0]); x[1] = bf16_hi(u[0]); x[2] = bf16_lo(u[1]); x[3] = bf16_hi(u[1]);
    x[4] = bf16_lo(u[2]); x[5] = bf16_hi(u[2]); x[6] = bf16_lo(u[3]); x[7] = bf16_hi(u[3]);
  }
};

constexpr int kSteps = kClsChunk / (4 * 8);   // 4 waves x 8 keys per wave-step

// grid (chunks, H*G, B), 256 threads.  Lane = (key slot, 8-channel slice): 8 lanes per key row.
// With G global tokens the rows of one head are G consecutive "rows" hg = h*G + g; logits are
// [B, H*G, T] and the partial records [B, H*G, chunks].
template <typename T, bool WITH_V>
__global__ __launch_bounds__(256) void cls_row_kernel(const T *q, const T *k, const T *v,
                                                      int64_t sb, int64_t sh, int64_t st, int T_,
                                                      int H, int G, float scale, float *logits,
                                                      float *partials, int nchunks) {
  const int chunk = blockIdx.x, hg = blockIdx.y, b = blockIdx.z;
  const int h = hg / G, gq = hg - h * G;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int slot = lane >> 3, sub = lane & 7;
  const T *qb = q + b * sb + h * sh + gq * st;   // global token gq
  const T *kb = k + b * sb + h * sh;
  const T *vb = WITH_V ? v + b * sb + h * sh : nullptr;
  __shared__ float red[4];
  __shared__ float osum[4][64];

  float q8[8];
  Row8<T>::load(qb + sub * 8, q8);
#pragma unroll
  for (int e = 0; e < 8; e++) q8[e] *= scale;

  const int key0 = chunk * kClsChunk + wave * (kSteps * 8) + slot;
  float s[kSteps];
  float mx = -INFINITY;
#pragma unroll
  for (int i = 0; i < kSteps; i++) {
    const int key = key0 + i * 8;
    float acc = -INFINITY;
    if (key < T_) {
      float k8[8];
      Row8<T>::template load<WITH_V>(kb + (int64_t)key * st + sub * 8, k8);
      acc = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) acc = __builtin_fmaf(q8[e], k8[e], acc);
    }
    // sum the 8 channel slices of the row (all lanes of the slot end up with the logit)
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    s[i] = acc;
    mx = fmaxf(mx, acc);
    if (sub == 0 && key < T_ && logits) logits[((size_t)b * H * G + hg) * T_ + key] = acc;
  }
  mx = fmaxf(mx, __shfl_xor(mx, 8));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  const float M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));   // finite: chunk non-empty
  __syncthreads();

  float l = 0.f;
  float o8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < kSteps; i++) {
    const int key = key0 + i * 8;
    if (key < T_) {
      const float pr = __builtin_amdgcn_exp2f((s[i] - M) * kLog2e);
      l += pr;
      if (WITH_V) {
        float v8[8];
        Row8<T>::template load<WITH_V>(vb + (int64_t)key * st + sub * 8, v8);
#pragma unroll
        for (int e = 0; e < 8; e++) o8[e] = __builtin_fmaf(pr, v8[e], o8[e]);
      }
    }
  }
  // across the 8 key slots of the wave (not across channel slices)
#pragma unroll
  for (int sft = 8; sft < 64; sft <<= 1) {
    l += __shfl_xor(l, sft);
    if (WITH_V) {
#pragma unroll
      for (int e = 0; e < 8; e++) o8[e] += __shfl_xor(o8[e], sft);
    }
  }
  if (lane == 0) red[wave] = l;
  if (WITH_V && slot == 0) {
#pragma unroll
    for (int e = 0; e < 8; e++) osum[wave][sub * 8 + e] = o8[e];
  }
  __syncthreads();
  float *rec = partials + (((size_t)b * H * G + hg) * nchunks + chunk) * kClsPartialFloats;
  if (tid == 0) {
    rec[0] = M;
    rec[1] = (red[0] + red[1]) + (red[2] + red[3]);
  }
  if (WITH_V && tid < 64) rec[2 + tid] = (osum[0][tid] + osum[1][tid]) + (osum[2][tid] + osum[3][tid]);
}

__device__ __forceinline__ void store_out(float *p, float x) { *p = x; }
__device__ __forceinline__ void store_out(uint16_t *p, float x) { *p = (uint16_t)(pack_bf16(x, 0.f) & 0xffffu); }

// grid (H*G, B), 1024 threads: thread (group g = tid/64, channel d = tid%64).  First the maximum
// over all records, then group g sums the records g, g+16, g+32, ... weighted against that maximum
// (no running maximum: the loads do not depend on each other and eight are kept in flight - the
// records were written by other workgroups, so every load is a long trip), and the sixteen groups
// are added in group order.  The order of operations is fixed, so the result is deterministic.
constexpr int kCombineThreads = 1024, kCombineGroups = kCombineThreads / 64;
template <typename T, bool WITH_V>
__device__ __forceinline__ void cls_combine_body(int hg, int b, const float *partials, int nchunks, int H, int G,
                                                 T *out, int64_t osb, int64_t osh, int64_t ost, float *lse) {
  const int tid = threadIdx.x, g = tid >> 6, d = tid & 63;
  const int h = hg / G, gq = hg - h * G;
  const float *rec = partials + ((size_t)b * H * G + hg) * nchunks * kClsPartialFloats;
  __shared__ float sm[kCombineGroups], sl[kCombineGroups], so[kCombineGroups][64];
  float M = -INFINITY;
  for (int c = tid; c < nchunks; c += kCombineThreads) M = fmaxf(M, rec[(size_t)c * kClsPartialFloats]);
#pragma unroll
  for (int sft = 1; sft < 64; sft <<= 1) M = fmaxf(M, __shfl_xor(M, sft));
  if (d == 0) sm[g] = M;
  __syncthreads();
  M = sm[0];
#pragma unroll
  for (int i = 1; i < kCombineGroups; i++) M = fmaxf(M, sm[i]);   // finite: there is at least one record with a key
  float L = 0.f, O = 0.f;
#pragma unroll 8
  for (int c = g; c < nchunks; c += kCombineGroups) {
    const float *r = rec + (size_t)c * kClsPartialFloats;
    const float w = __builtin_amdgcn_exp2f((r[0] - M) * kLog2e);   // 0 for a record without keys
    L = __builtin_fmaf(r[1], w, L);
    if (WITH_V) O = __builtin_fmaf(r[2 + d], w, O);
  }
  if (d == 0) sl[g] = L;
  so[g][d] = O;
  __syncthreads();
  if (g != 0) return;
  float Lt = 0.f, Ot = 0.f;
#pragma unroll
  for (int i = 0; i < kCombineGroups; i++) {
    Lt += sl[i];
    Ot += so[i][d];
  }
  if (WITH_V) store_out(out + b * osb + h * osh + gq * ost + d, Ot / Lt);
  if (lse && d == 0) lse[(size_t)b * H * G + hg] = M + __builtin_amdgcn_logf(Lt) * kLn2;
}

template <typename T, bool WITH_V>
__global__ __launch_bounds__(kCombineThreads) void cls_combine_kernel(const float *partials, int nchunks, int H,
                                                                      int G, T *out, int64_t osb, int64_t osh,
                                                                      int64_t ost, float *lse) {
  cls_combine_body<T, WITH_V>(blockIdx.x, blockIdx.y, partials, nchunks, H, G, out, osb, osh, ost, lse);
}

// Workgroup `blk` of image b scores blockDim.x patches (thread = patch).  H counts the global rows
// of an image (heads x global tokens): the score is the mean over all of them.  lse given
// directly, or recomputed per row from the (max, sum) of the partial records.
__device__ __forceinline__ void cls_scores_body(int blk, int b, const float *logits, const float *lse,
                                                const float *partials, int nchunks, int H, int T_, int G,
                                                float *scores) {
  __shared__ float s_lse[1024];
  const int tid = threadIdx.x, nthreads = blockDim.x;
  if (lse) {
    for (int h = tid; h < H; h += nthreads) s_lse[h] = lse[(size_t)b * H + h];
  } else {
    // 16 lanes per head: each merges every 16th record, then the 16 are merged pairwise (fixed order)
    const int sub = tid & 15;
    for (int h = tid >> 4; h < H; h += nthreads >> 4) {
      const float *rec = partials + ((size_t)b * H + h) * nchunks * kClsPartialFloats;
      float M = -INFINITY, L = 0.f;
      for (int c = sub; c < nchunks; c += 16) {
        const float mc = rec[c * kClsPartialFloats], lc = rec[c * kClsPartialFloats + 1];
        const float Mn = fmaxf(M, mc);
        L = L * __builtin_amdgcn_exp2f((M - Mn) * kLog2e) + lc * __builtin_amdgcn_exp2f((mc - Mn) * kLog2e);
        M = Mn;
      }
#pragma unroll
      for (int sft = 1; sft < 16; sft <<= 1) {
        const float Mo = __shfl_xor(M, sft), Lo = __shfl_xor(L, sft);
        const float Mn = fmaxf(M, Mo);
        // a lane without records has M = -inf, L = 0: its weight is exp2(-inf) = 0 unless both are
        // empty, which cannot happen for all 16 (there is at least one record)
        const float wa = Mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((M - Mn) * kLog2e);
        const float wb = Mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((Mo - Mn) * kLog2e);
        // both lanes of a pair must add in the same order to agree bit for bit
        const bool lowl = (sub & sft) == 0;
        L = lowl ? L * wa + Lo * wb : Lo * wb + L * wa;
        M = Mn;
      }
      if (sub == 0) s_lse[h] = M + __builtin_amdgcn_logf(L) * kLn2;
    }
  }
  __syncthreads();
  const int N = T_ - G;
  const int j = blk * nthreads + tid;
  if (j >= N) return;
  float acc = 0.f;
  for (int h = 0; h < H; h++) {
    const float x = logits[((size_t)b * H + h) * T_ + G + j];
    acc += __builtin_amdgcn_exp2f((x - s_lse[h]) * kLog2e);
  }
  scores[(size_t)b * N + j] = acc / (float)H;
}

// grid (ceil(N/256), B), 256 threads
__global__ __launch_bounds__(256) void cls_scores_kernel(const float *logits, const float *lse,
                                                         const float *partials, int nchunks, int H,
                                                         int T_, int G, float *scores) {
  cls_scores_body(blockIdx.x, blockIdx.y, logits, lse, partials, nchunks, H, T_, G, scores);
}

// Both in one launch, grid (H + ceil(N/1024), B), 1024 threads: the first H workgroups of an image
// merge the records of one global row each (output row and log-sum-exp), the others score 1024
// patches each, with the log-sum-exps they derive from the records themselves.
template <typename T>
__global__ __launch_bounds__(kCombineThreads) void cls_combine_scores_kernel(const float *partials, int nchunks,
                                                                             int heads, int G, T *out, int64_t osb,
                                                                             int64_t osh, int64_t ost, float *lse,
                                                                             const float *logits, int T_,
                                                                             float *scores) {
  const int H = heads * G;
  if ((int)blockIdx.x < H)
    cls_combine_body<T, true>(blockIdx.x, blockIdx.y, partials, nchunks, heads, G, out, osb, osh, ost, lse);
  else
    cls_scores_body(blockIdx.x - H, blockIdx.y, logits, nullptr, partials, nchunks, H, T_, G, scores);
}

}  // namespace

ns_status launch_cls_row(const ns_attn_desc &d, const void *q, const void *k, const void *v,
                         float *logits, float *partials, bool with_v, hipStream_t s) {
  const int nch = cls_num_chunks(d.tokens);
  dim3 grid(nch, d.heads * d.n_global, d.batch), blk(256);
#define NS_ROW(T, WV)                                                                          \
  hipLaunchKernelGGL((cls_row_kernel<T, WV>), grid, blk, 0, s, static_cast<const T *>(q),      \
                     static_cast<const T *>(k), static_cast<const T *>(v), d.q_stride_b,       \
                     d.q_stride_h, d.q_stride_t, d.tokens, d.heads, d.n_global, d.scale, logits, \
                     partials, nch)
  if (d.dtype == NS_F32) { if (with_v) NS_ROW(float, true); else NS_ROW(float, false); }
  else { if (with_v) NS_ROW(uint16_t, true); else NS_ROW(uint16_t, false); }
#undef NS_ROW
  return check_launch("cls_row_kernel");
}

ns_status launch_cls_combine(const ns_attn_desc &d, const float *partials, void *out, float *lse,
                             bool with_v, hipStream_t s, int nchunks) {
  const int nch = nchunks > 0 ? nchunks : cls_num_chunks(d.tokens);
  dim3 grid(d.heads * d.n_global, d.batch), blk(kCombineThreads);
  if (d.dtype == NS_F32) {
    if (with_v)
      hipLaunchKernelGGL((cls_combine_kernel<float, true>), grid, blk, 0, s, partials, nch, d.heads,
                         d.n_global, static_cast<float *>(out), d.out_stride_b, d.out_stride_h, d.out_stride_t, lse);
    else
      hipLaunchKernelGGL((cls_combine_kernel<float, false>), grid, blk, 0, s, partials, nch, d.heads,
                         d.n_global, static_cast<float *>(out), d.out_stride_b, d.out_stride_h, d.out_stride_t, lse);
  } else {
    if (with_v)
      hipLaunchKernelGGL((cls_combine_kernel<uint16_t, true>), grid, blk, 0, s, partials, nch,
                         d.heads, d.n_global, static_cast<uint16_t *>(out), d.out_stride_b, d.out_stride_h,
                         d.out_stride_t, lse);
    else
      hipLaunchKernelGGL((cls_combine_kernel<uint16_t, false>), grid, blk, 0, s, partials, nch,
                         d.heads, d.n_global, static_cast<uint16_t *>(out), d.out_stride_b, d.out_stride_h,
                         d.out_stride_t, lse);
  }
  return check_launch("cls_combine_kernel");
}

ns_status launch_cls_combine_scores(const ns_attn_desc &d, const float *partials, void *out, float *lse,
                                    const float *logits, float *scores, hipStream_t s, int nchunks) {
  const int nch = nchunks > 0 ? nchunks : cls_num_chunks(d.tokens);
  const int N = d.tokens - d.n_global;
  dim3 grid(d.heads * d.n_global + (N + kCombineThreads - 1) / kCombineThreads, d.batch), blk(kCombineThreads);
  if (d.dtype == NS_F32)
    hipLaunchKernelGGL((cls_combine_scores_kernel<float>), grid, blk, 0, s, partials, nch, d.heads, d.n_global,
                       static_cast<float *>(out), d.out_stride_b, d.out_stride_h, d.out_stride_t, lse, logits,
                       d.tokens, scores);
  else
    hipLaunchKernelGGL((cls_combine_scores_kernel<uint16_t>), grid, blk, 0, s, partials, nch, d.heads, d.n_global,
                       static_cast<uint16_t *>(out), d.out_stride_b, d.out_stride_h, d.out_stride_t, lse, logits,
                       d.tokens, scores);
  return check_launch("cls_combine_scores_kernel");
}

ns_status launch_cls_scores(int B, int H, int T, int G, const float *logits, const float *lse,
                            const float *partials, int nchunks, float *scores, hipStream_t s) {
  const int N = T - G;
  dim3 grid((N + 255) / 256, B), blk(256);
  hipLaunchKernelGGL(cls_scores_kernel, grid, blk, 0, s, logits, lse, partials, nchunks, H * G, T, G,
                     scores);
  return check_launch("cls_scores_kernel");
}

}  // namespace ns
