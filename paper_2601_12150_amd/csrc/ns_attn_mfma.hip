// bf16 MFMA neighbourhood attention for patch queries on the full grid (gfx950).
//
// Pattern: paper, "Memory-Efficiency Optimization" -- a patch query sees the patches of the
// 3x3 token blocks around its own block and the global token.  With b*b a multiple of 64 a
// block splits into tiles of 64 tokens (64/b grid rows of b tokens) and every (query tile,
// key tile) pair of neighbouring blocks is a dense 64x64 problem: no masking inside tiles.
//
// One wave owns one query tile for its whole life and walks the key tiles of the <= 9
// neighbour blocks.  Everything is computed transposed so that all per-query state lives
// in that query's lane pair:
//   S^T[key][query]  = K_tile (A operand) x Q^T (B operand)         v_mfma_f32_32x32x16_bf16
//   O^T[chan][query] += V_tile^T (A operand) x P^T (B operand)
// The accumulator layout of S^T (lane = query column, 16 key rows per 32x32 tile) is, after
// exp and bf16 packing, already the B-operand layout of the second product, so P never
// leaves registers.  K fragments are read straight from global memory (the contraction runs
// over channels, which are contiguous); V needs its contraction index (keys) transposed into
// lanes, which ds_read_b64_tr_b16 does out of a row-major LDS copy of the tile.
// The global token initialises the online-softmax state (m = its logit, l = 1, O = v_0).
#include "ns_common.h"

namespace ns {

namespace {

struct MfmaParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float c;             // scale * log2(e)
  int grid_w, nbh, nbw;
  int heads;
  int wgs_per_image;   // workgroups per (batch, head)
  int tiles_per_image; // query tiles per (batch, head)
  int total_wgs;
};

__device__ __forceinline__ float half_swap_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// LOG2B: log2 of the block side (3 -> 8x8 blocks = 1 tile, 4 -> 16x16 blocks = 4 tiles).
template <int LOG2B>
__global__ __launch_bounds__(256) void attn_mfma_kernel(MfmaParams p) {
  constexpr int B_ = 1 << LOG2B;             // block side
  constexpr int TPB = (B_ * B_) / 64;        // tiles per block
  constexpr int TROWS = 64 / B_;             // grid rows per tile
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int l32 = lane & 31, hh = lane >> 5;

  // XCD-aware order: consecutive workgroup ids go round-robin over the 8 XCDs, so give each
  // XCD a contiguous range of logical workgroups (whole head-images share one L2).
  int bid = blockIdx.x;
  if ((p.total_wgs & 7) == 0) bid = (bid & 7) * (p.total_wgs >> 3) + (bid >> 3);
  const int img = bid / p.wgs_per_image;
  const int qt = (bid % p.wgs_per_image) * 4 + wave;
  if (qt >= p.tiles_per_image) return;       // no workgroup barriers below
  const int b = img / p.heads, h = img % p.heads;
  const int blk = qt / TPB, qsub = qt % TPB;
  const int R = blk / p.nbw, C = blk % p.nbw;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *vlds = smem + wave * 8192;  // this wave's V tile, row-major [key][64] bf16

  const uint16_t *qb = p.q + b * p.qsb + h * p.qsh;
  const uint16_t *kb = p.k + b * p.qsb + h * p.qsh;
  const uint16_t *vb = p.v + b * p.qsb + h * p.qsh;

  // token offset (in tokens) of element i of a tile relative to the tile's first token
  auto tile_off = [&](int i) { return (i >> LOG2B) * p.grid_w + (i & (B_ - 1)); };
  auto tile_base = [&](int R2, int C2, int sub) {
    return 1 + (R2 * B_ + sub * TROWS) * p.grid_w + C2 * B_;
  };

  // ---- Q as B operand: lane (query l32 + 32*nt, half hh) holds channels 32*hh + 8*s + j
  bf16x8 qf[2][4];
  const int qbase = tile_base(R, C, qsub);
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const uint16_t *row = qb + (int64_t)(qbase + tile_off(l32 + 32 * nt)) * p.qst + 32 * hh;
#pragma unroll
    for (int s = 0; s < 4; s++) qf[nt][s] = *reinterpret_cast<const bf16x8 *>(row + 8 * s);
  }

  // ---- state initialised by the global token (key 0)
  float m[2], l[2];
  f32x16 o[2][2];   // [dt][nt]: channel rows 32*dt + 8*(i/4) + 4*hh + i%4, query column
  {
    bf16x8 k0[4];
#pragma unroll
    for (int s = 0; s < 4; s++) k0[s] = *reinterpret_cast<const bf16x8 *>(kb + 32 * hh + 8 * s);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      float acc = 0.f;
#pragma unroll
      for (int s = 0; s < 4; s++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc = __builtin_fmaf((float)qf[nt][s][j], (float)k0[s][j], acc);
      acc = half_swap_sum(acc);
      m[nt] = acc * p.c;
      l[nt] = hh == 0 ? 1.f : 0.f;
    }
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        const bf16x4 v4 = *reinterpret_cast<const bf16x4 *>(vb + 32 * dt + 8 * ig + 4 * hh);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[dt][0][4 * ig + e] = (float)v4[e];
          o[dt][1][4 * ig + e] = (float)v4[e];
        }
      }
  }

  // per-lane addressing that does not depend on the key tile
  int koff[2];
#pragma unroll
  for (int mt = 0; mt < 2; mt++) koff[mt] = tile_off(l32 + 32 * mt);
  const int vchunk = lane & 7;
  int voff[8], vlds_w[8];
#pragma unroll
  for (int it = 0; it < 8; it++) {
    const int key = it * 8 + (lane >> 3);
    voff[it] = tile_off(key);
    vlds_w[it] = key * 128 + ((vchunk * 16) ^ (((key >> 1) & 1) << 6));
  }
  // transposed reads: 16-lane group g, source lane s: row key0 + s/4, channels dbase + 4*(s%4)
  int vlds_r[2];   // [which 4-key group]; add ks*16*128 bytes and dt*64 bytes (pre-swizzle)
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);     // + 16*ks, which keeps (key>>1)&1
      vlds_r[half] = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
    }
  }

  for (int nb = 0; nb < 9; nb++) {
    const int R2 = R + nb / 3 - 1, C2 = C + nb % 3 - 1;
    if (R2 < 0 || R2 >= p.nbh || C2 < 0 || C2 >= p.nbw) continue;
#pragma unroll 1
    for (int sub = 0; sub < TPB; sub++) {
      const int kbase = tile_base(R2, C2, sub);
      // ---- K fragments (A operand) straight from global memory
      bf16x8 kf[2][4];
#pragma unroll
      for (int mt = 0; mt < 2; mt++) {
        const uint16_t *row = kb + (int64_t)(kbase + koff[mt]) * p.qst + 32 * hh;
#pragma unroll
        for (int s = 0; s < 4; s++) kf[mt][s] = *reinterpret_cast<const bf16x8 *>(row + 8 * s);
      }
      // ---- V tile: global -> registers (written to LDS after the first product)
      uint4 vr[8];
#pragma unroll
      for (int it = 0; it < 8; it++)
        vr[it] = *reinterpret_cast<const uint4 *>(vb + (int64_t)(kbase + voff[it]) * p.qst + vchunk * 8);

      // ---- S^T = K Q^T
      f32x16 st[2][2];
#pragma unroll
      for (int mt = 0; mt < 2; mt++)
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
          f32x16 acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < 4; s++)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][s], qf[nt][s], acc, 0, 0, 0);
          st[mt][nt] = acc;
        }

      // ---- V tile into LDS (this wave's private slice; previous tile's reads are done)
#pragma unroll
      for (int it = 0; it < 8; it++) *reinterpret_cast<uint4 *>(vlds + vlds_w[it]) = vr[it];

      // ---- online softmax, per query column
      bf16x8 pf[2][4];   // [nt][ks]: B operand of the second product
#pragma unroll
      for (int nt = 0; nt < 2; nt++) {
        float mx = st[0][nt][0];
#pragma unroll
        for (int i = 1; i < 16; i++) mx = fmaxf(mx, st[0][nt][i]);
#pragma unroll
        for (int i = 0; i < 16; i++) mx = fmaxf(mx, st[1][nt][i]);
        mx = half_swap_max(mx);
        const float m_new = fmaxf(m[nt], mx * p.c);
        const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
        m[nt] = m_new;
        float ls = 0.f;
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
#pragma unroll
          for (int i = 0; i < 16; i += 2) {
            const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[mt][nt][i], p.c, -m_new));
            const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(st[mt][nt][i + 1], p.c, -m_new));
            ls += p0 + p1;
            const bf16x2 pk = __builtin_bit_cast(bf16x2, pack_bf16(p0, p1));
            pf[nt][2 * mt + (i >> 3)][i & 7] = pk[0];
            pf[nt][2 * mt + (i >> 3)][(i & 7) + 1] = pk[1];
          }
        l[nt] = __builtin_fmaf(l[nt], alpha, ls);
        if (__any(alpha != 1.f)) {
#pragma unroll
          for (int dt = 0; dt < 2; dt++)
#pragma unroll
            for (int i = 0; i < 16; i++) o[dt][nt][i] *= alpha;
        }
      }

      // ---- O^T += V^T P^T
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int ks = 0; ks < 4; ks++)
#pragma unroll
        for (int dt = 0; dt < 2; dt++) {
          const int sw = dt * 64;   // second channel tile: +64 bytes, commutes with the bit-6 swizzle
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4 __attribute__((address_space(3))) *)(vlds + ((vlds_r[0] + ks * 2048) ^ sw)));
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
              (s16x4 __attribute__((address_space(3))) *)(vlds + ((vlds_r[1] + ks * 2048) ^ sw)));
          bf16x8 vf;
          const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
#pragma unroll
          for (int e = 0; e < 4; e++) { vf[e] = lo4[e]; vf[4 + e] = hi4[e]; }
#pragma unroll
          for (int nt = 0; nt < 2; nt++)
            o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[nt][ks], o[dt][nt], 0, 0, 0);
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
  }

  // ---- normalise and store: lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3
  uint16_t *ob = p.out + b * p.osb + h * p.osh;
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const float inv = 1.f / half_swap_sum(l[nt]);
    uint16_t *row = ob + (int64_t)(qbase + tile_off(l32 + 32 * nt)) * p.ost + 4 * hh;
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        uint2 u = {pack_bf16(o[dt][nt][4 * ig] * inv, o[dt][nt][4 * ig + 1] * inv),
                   pack_bf16(o[dt][nt][4 * ig + 2] * inv, o[dt][nt][4 * ig + 3] * inv)};
        *reinterpret_cast<uint2 *>(row + 32 * dt + 8 * ig) = u;
      }
  }
}

}  // namespace

bool mfma_attn_supported(const ns_attn_desc &d) {
  return d.dtype == NS_BF16 && d.head_dim == 64 && d.radius == 1 && d.n_global == 1 &&
         d.coords == nullptr && (d.block == 8 || d.block == 16) && d.grid_h % d.block == 0 &&
         d.grid_w % d.block == 0 && d.scale > 0.f;
}

ns_status launch_attn_mfma(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  MfmaParams p;
  p.q = static_cast<const uint16_t *>(a.q);
  p.k = static_cast<const uint16_t *>(a.k);
  p.v = static_cast<const uint16_t *>(a.v);
  p.out = static_cast<uint16_t *>(a.out);
  p.qsb = d.q_stride_b; p.qsh = d.q_stride_h; p.qst = d.q_stride_t;
  p.osb = d.out_stride_b; p.osh = d.out_stride_h; p.ost = d.out_stride_t;
  p.c = d.scale * kLog2e;
  p.grid_w = d.grid_w;
  p.nbh = d.grid_h / d.block;
  p.nbw = d.grid_w / d.block;
  p.heads = d.heads;
  p.tiles_per_image = p.nbh * p.nbw * (d.block * d.block / 64);
  p.wgs_per_image = (p.tiles_per_image + 3) / 4;
  const long long total = (long long)p.wgs_per_image * d.heads * d.batch;
  if (total > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "launch grid too large");
  p.total_wgs = (int)total;
  const size_t lds = 4 * 8192;
  if (d.block == 8)
    hipLaunchKernelGGL(attn_mfma_kernel<3>, dim3(p.total_wgs), dim3(256), lds, a.stream, p);
  else
    hipLaunchKernelGGL(attn_mfma_kernel<4>, dim3(p.total_wgs), dim3(256), lds, a.stream, p);
  return check_launch("attn_mfma_kernel");
}

}  // namespace ns
