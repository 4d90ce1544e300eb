// Shape-generic neighbourhood attention for patch queries (any block size, ragged blocks,
// pruned sequences, fp32 or bf16 storage) and the block-list builder for pruned sequences.
//
// Pattern: paper, "Memory-Efficiency Optimization" -- a patch query sees the patches of the
// 3x3 blocks around its own block plus the global token.  This kernel is the fallback for
// shapes the MFMA kernel does not take; it computes in fp32 on the vector ALU.
//
// One workgroup (4 waves) owns up to 64 queries of one block; lane = query.  The four waves
// split the key chunks (16 keys each) round-robin, each keeping its own online-softmax state,
// and merge through LDS in a fixed order, so results are deterministic.
#include "ns_common.h"

namespace ns {

namespace {

constexpr int kChunk = 16;   // keys staged per step and wave
constexpr int kD = 64;       // head_dim

struct GenericParams {
  const void *q, *k, *v;
  void *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float scale_log2e;
  int tiles_per_block;
  BlockGeom g;
};

template <typename T> struct Elem;
template <> struct Elem<float> {
  __device__ static f32x4 load4(const float *p) { return *reinterpret_cast<const f32x4 *>(p); }
  __device__ static void store4(float *p, f32x4 v) { *reinterpret_cast<f32x4 *>(p) = v; }
};
template <> struct Elem<uint16_t> {
  __device__ static f32x4 load4(const uint16_t *p) {
    uint2 u = *reinterpret_cast<const uint2 *>(p);
    f32x4 r = {bf16_lo(u.x), bf16_hi(u.x), bf16_lo(u.y), bf16_hi(u.y)};
    return r;
  }
  __device__ static void store4(uint16_t *p, f32x4 v) {
    uint2 u = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
    *reinterpret_cast<uint2 *>(p) = u;
  }
};

template <typename T>
__global__ __launch_bounds__(256) void attn_generic_kernel(GenericParams p) {
  const BlockGeom &g = p.g;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int blk = blockIdx.x / p.tiles_per_block, tile = blockIdx.x % p.tiles_per_block;
  const int R = blk / g.nbw, C = blk % g.nbw;
  const int h = blockIdx.y, b = blockIdx.z;
  const int cnt = block_count(g, b, R, C);
  const int q0 = tile * 64;
  if (q0 >= cnt) return;

  __shared__ float Ks[4][kChunk][kD];
  __shared__ float Vs[4][kChunk][kD];
  __shared__ float ml[4][2][64];

  const T *qb = static_cast<const T *>(p.q) + b * p.qsb + h * p.qsh;
  const T *kb = static_cast<const T *>(p.k) + b * p.qsb + h * p.qsh;
  const T *vb = static_cast<const T *>(p.v) + b * p.qsb + h * p.qsh;

  const bool valid = q0 + lane < cnt;
  const int qtok = block_token(g, b, R, C, valid ? q0 + lane : q0);
  float qr[kD], o[kD];
#pragma unroll
  for (int d = 0; d < kD; d += 4) {
    f32x4 t = Elem<T>::load4(qb + (int64_t)qtok * p.qst + d);
#pragma unroll
    for (int e = 0; e < 4; e++) { qr[d + e] = t[e] * p.scale_log2e; o[d + e] = 0.f; }
  }
  float m = -INFINITY, l = 0.f;

  int cidx = 0;
  for (int nb = -1; nb < 9; nb++) {
    int R2 = 0, C2 = 0, n;
    if (nb < 0) {
      n = g.n_global;
    } else {
      R2 = R + nb / 3 - 1;
      C2 = C + nb % 3 - 1;
      if (R2 < 0 || R2 >= g.nbh || C2 < 0 || C2 >= g.nbw) continue;
      n = block_count(g, b, R2, C2);
    }
    for (int c0 = 0; c0 < n; c0 += kChunk, cidx++) {
      if ((cidx & 3) != wave) continue;
      const int nk = min(kChunk, n - c0);
      // stage up to 16 key and value rows as fp32 in this wave's LDS slice
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int key = (lane >> 4) + 4 * i, quad = lane & 15;
        if (key < nk) {
          const int tok = nb < 0 ? c0 + key : block_token(g, b, R2, C2, c0 + key);
          f32x4 kk = Elem<T>::load4(kb + (int64_t)tok * p.qst + quad * 4);
          f32x4 vv = Elem<T>::load4(vb + (int64_t)tok * p.qst + quad * 4);
          *reinterpret_cast<f32x4 *>(&Ks[wave][key][quad * 4]) = kk;
          *reinterpret_cast<f32x4 *>(&Vs[wave][key][quad * 4]) = vv;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

      float s[kChunk];
      float cm = -INFINITY;
#pragma unroll
      for (int key = 0; key < kChunk; key++) {
        float acc = 0.f;
        if (key < nk) {
#pragma unroll
          for (int d = 0; d < kD; d += 4) {
            f32x4 kk = *reinterpret_cast<const f32x4 *>(&Ks[wave][key][d]);
            acc = __builtin_fmaf(qr[d], kk[0], acc);
            acc = __builtin_fmaf(qr[d + 1], kk[1], acc);
            acc = __builtin_fmaf(qr[d + 2], kk[2], acc);
            acc = __builtin_fmaf(qr[d + 3], kk[3], acc);
          }
        } else {
          acc = -INFINITY;
        }
        s[key] = acc;
        cm = fmaxf(cm, acc);
      }
      const float m_new = fmaxf(m, cm);           // finite: the chunk holds at least one key
      const float alpha = __builtin_amdgcn_exp2f(m - m_new);
      l *= alpha;
#pragma unroll
      for (int d = 0; d < kD; d++) o[d] *= alpha;
#pragma unroll
      for (int key = 0; key < kChunk; key++) {
        if (key < nk) {
          const float pr = __builtin_amdgcn_exp2f(s[key] - m_new);
          l += pr;
#pragma unroll
          for (int d = 0; d < kD; d += 4) {
            f32x4 vv = *reinterpret_cast<const f32x4 *>(&Vs[wave][key][d]);
            o[d] = __builtin_fmaf(pr, vv[0], o[d]);
            o[d + 1] = __builtin_fmaf(pr, vv[1], o[d + 1]);
            o[d + 2] = __builtin_fmaf(pr, vv[2], o[d + 2]);
            o[d + 3] = __builtin_fmaf(pr, vv[3], o[d + 3]);
          }
        }
      }
      m = m_new;
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }

  // merge the four waves' states: weights first, then the value sums in wave order
  ml[wave][0][lane] = m;
  ml[wave][1][lane] = l;
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; w++) M = fmaxf(M, ml[w][0][lane]);
  float L = 0.f;
#pragma unroll
  for (int w = 0; w < 4; w++) L += ml[w][1][lane] * __builtin_amdgcn_exp2f(ml[w][0][lane] - M);
  const float f = __builtin_amdgcn_exp2f(m - M) / L;   // 0 for a wave that saw no key
  float *acc = &Ks[0][0][0];                           // reused as [d][lane] fp32 (16 KB)
  for (int w = 0; w < 4; w++) {
    if (wave == w) {
#pragma unroll
      for (int d = 0; d < kD; d++) {
        const float t = f * o[d];
        acc[d * 64 + lane] = (w == 0) ? t : acc[d * 64 + lane] + t;
      }
    }
    __syncthreads();
  }
  T *ob = static_cast<T *>(p.out) + b * p.osb + h * p.osh;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int idx = tid + 256 * i, ql = idx >> 4, quad = idx & 15;
    if (q0 + ql < cnt) {
      const int tok = block_token(g, b, R, C, q0 + ql);
      f32x4 t = {acc[(quad * 4) * 64 + ql], acc[(quad * 4 + 1) * 64 + ql],
                 acc[(quad * 4 + 2) * 64 + ql], acc[(quad * 4 + 3) * 64 + ql]};
      Elem<T>::store4(ob + (int64_t)tok * p.ost + quad * 4, t);
    }
  }
}

// Pruned sequence: bucket the surviving patch tokens by block, preserving sequence order.
// grid (nblocks, B); each workgroup scans the image's coordinate list for its own block.
__global__ __launch_bounds__(256) void block_lists_kernel(const int32_t *coords, int n_patch,
                                                          int n_global, int grid_h, int grid_w,
                                                          int block, int nbw, int nblocks, int cap,
                                                          int32_t *lists, int32_t *counts) {
  const int blk = blockIdx.x, b = blockIdx.y;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  __shared__ int wcnt[4];
  const int32_t *cb = coords + (size_t)b * n_patch;
  int32_t *lb = lists + ((size_t)b * nblocks + blk) * cap;
  int running = 0;
  for (int base = 0; base < n_patch; base += 256) {
    const int j = base + tid;
    bool match = false;
    if (j < n_patch) {
      const uint32_t pc = (uint32_t)cb[j];
      const int r = (int)(pc >> 16), c = (int)(pc & 0xffffu);
      match = r < grid_h && c < grid_w && (r / block) * nbw + (c / block) == blk;
    }
    const unsigned long long bal = __ballot(match);
    if (lane == 0) wcnt[wave] = __popcll(bal);
    __syncthreads();
    int off = running;
    for (int w = 0; w < wave; w++) off += wcnt[w];
    off += __popcll(bal & ((1ull << lane) - 1ull));
    if (match && off < cap) lb[off] = n_global + j;
    running += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
    __syncthreads();
  }
  if (tid == 0) counts[(size_t)b * nblocks + blk] = min(running, cap);
}

// Complete grid: the same lists in closed form (raster order inside a block; the last block of a
// row or column is short when the block side does not divide the grid).  grid (nblocks, B).
__global__ __launch_bounds__(256) void grid_lists_kernel(int n_global, int grid_h, int grid_w, int block,
                                                         int nbw, int nblocks, int cap, int32_t *lists,
                                                         int32_t *counts) {
  const int blk = blockIdx.x, b = blockIdx.y;
  const int R = blk / nbw, C = blk % nbw;
  const int bh = min(block, grid_h - R * block), bw = min(block, grid_w - C * block);
  const int cnt = bh * bw;
  int32_t *lb = lists + ((size_t)b * nblocks + blk) * cap;
  for (int s = threadIdx.x; s < cnt; s += 256)
    lb[s] = n_global + (R * block + s / bw) * grid_w + C * block + s % bw;
  if (threadIdx.x == 0) counts[(size_t)b * nblocks + blk] = cnt;
}

}  // namespace

ns_status launch_grid_lists(const ns_attn_desc &d, int32_t *lists, int32_t *counts, hipStream_t s) {
  const int nbh = (d.grid_h + d.block - 1) / d.block, nbw = (d.grid_w + d.block - 1) / d.block;
  dim3 grid(nbh * nbw, d.batch);
  hipLaunchKernelGGL(grid_lists_kernel, grid, dim3(256), 0, s, d.n_global, d.grid_h, d.grid_w, d.block, nbw,
                     nbh * nbw, d.block * d.block, lists, counts);
  return check_launch("grid_lists_kernel");
}

ns_status launch_block_lists(const ns_attn_desc &d, int32_t *lists, int32_t *counts, hipStream_t s) {
  const int nbh = (d.grid_h + d.block - 1) / d.block, nbw = (d.grid_w + d.block - 1) / d.block;
  dim3 grid(nbh * nbw, d.batch);
  hipLaunchKernelGGL(block_lists_kernel, grid, dim3(256), 0, s, d.coords, d.tokens - d.n_global,
                     d.n_global, d.grid_h, d.grid_w, d.block, nbw, nbh * nbw, d.block * d.block,
                     lists, counts);
  return check_launch("block_lists_kernel");
}

ns_status launch_attn_generic(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  GenericParams p;
  p.q = a.q; p.k = a.k; p.v = a.v; p.out = a.out;
  p.qsb = d.q_stride_b; p.qsh = d.q_stride_h; p.qst = d.q_stride_t;
  p.osb = d.out_stride_b; p.osh = d.out_stride_h; p.ost = d.out_stride_t;
  p.scale_log2e = d.scale * kLog2e;
  p.g = a.geom;
  p.tiles_per_block = (a.geom.cap + 63) / 64;
  const long long gx = (long long)a.geom.nbh * a.geom.nbw * p.tiles_per_block;
  if (gx > 0x7fffffffLL || d.heads > 65535 || d.batch > 65535)
    return fail(NS_ERR_UNSUPPORTED, "launch grid too large");
  dim3 grid((unsigned)gx, d.heads, d.batch);
  if (d.dtype == NS_F32)
    hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(256), 0, a.stream, p);
  else
    hipLaunchKernelGGL(attn_generic_kernel<uint16_t>, grid, dim3(256), 0, a.stream, p);
  return check_launch("attn_generic_kernel");
}

}  // namespace ns
