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



typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;

// LOG2B: log2 of the block side (3 -> 8x8 blocks = 1 tile, 4 -> 16x16 blocks = 4 tiles).
//
// A 64-key x 64-query tile is processed as four 32x32 sub-blocks (mt = key half, nt = query
// half), each with three stages:
//   A: S^T = K Q^T         4 MFMAs
//   B: p = exp2(c*S - m)   16 elements per lane on the vector ALU, row sums, bf16 pack
//   C: O^T += V^T P^T      4 MFMAs, V fragments transposed out of LDS
// The stages of consecutive sub-blocks are software-pipelined (A of sub-block j+1 and C of j-1
// around B of j), so that the matrix pipe and the vector ALU both have independent work in
// every stretch of the instruction stream.  The exponent reference m is the global token's
// logit and is NOT raised tile by tile: that makes B element-wise (no row maximum, no
// rescale of O^T, no branch).  It is exact as long as no weight overflows; the result is
// checked at the end and the query tile is redone with a running maximum if it did.
template <int LOG2B>
__global__ __launch_bounds__(256, 2) void attn_mfma_kernel(MfmaParams p) {
  constexpr int B_ = 1 << LOG2B;             // block side
  constexpr int TPB = (B_ * B_) / 64;        // tiles per block
  constexpr int TROWS = 64 / B_;             // grid rows per tile
  // the wave index is uniform by construction; telling the compiler keeps every quantity
  // derived from it (tile coordinates, trip counts, base addresses) in scalar registers
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
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
  unsigned char *vlds = smem + wave * 16384;  // two V tiles, row-major [key][64] bf16, swizzled

  const char *qb = reinterpret_cast<const char *>(p.q + b * p.qsb + h * p.qsh);
  const char *kb = reinterpret_cast<const char *>(p.k + b * p.qsb + h * p.qsh);
  const char *vb = reinterpret_cast<const char *>(p.v + b * p.qsb + h * p.qsh);
  const uint32_t rowB = (uint32_t)p.qst * 2u;          // bytes per token row step

  // token offset of element i of a tile relative to the tile's first token
  auto tile_off = [&](int i) { return (i >> LOG2B) * p.grid_w + (i & (B_ - 1)); };
  auto tile_base = [&](int R2, int C2, int sub) {
    return 1 + (R2 * B_ + sub * TROWS) * p.grid_w + C2 * B_;
  };

  // ---- Q as B operand: lane (query l32 + 32*nt, half hh) holds channels 32*hh + 8*s + j
  bf16x8 qf[2][4];
  const int qbase = tile_base(R, C, qsub);
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const char *row = qb + (size_t)(qbase + tile_off(l32 + 32 * nt)) * rowB + 64 * hh;
#pragma unroll
    for (int s = 0; s < 4; s++) qf[nt][s] = *reinterpret_cast<const bf16x8 *>(row + 16 * s);
  }

  // ---- per-lane byte offsets that do not depend on the key tile (one register each; the
  // per-fragment parts are wave-uniform and live in scalar registers)
  const uint32_t gridrowB = (uint32_t)p.grid_w * rowB;            // one grid row down
  const uint32_t koff = (uint32_t)tile_off(l32) * rowB + 64u * hh;
  const uint32_t kstep = (32 >> LOG2B) * gridrowB;                // keys 32..63 of a tile
  // V: 16-byte slot `lane` of LDS chunk `it` holds key it*8 + lane/8, stored chunk lane%8,
  // i.e. logical channel chunk (lane%8) ^ 4*((key>>1)&1)   (bank swizzle, see the reads);
  // (key>>1)&1 does not depend on `it`
  const uint32_t voff = (uint32_t)tile_off(lane >> 3) * rowB +
                        16u * ((lane & 7) ^ ((((lane >> 3) >> 1) & 1) << 2));
  auto vstep = [&](int it) {   // token offset of key it*8 relative to key 0, in bytes
    return LOG2B == 3 ? it * gridrowB : (it >> 1) * gridrowB + (it & 1) * 8u * rowB;
  };
  // transposed reads (ds_read_b64_tr_b16): within a 16-lane group, lane i receives element
  // i%4 of the 8-byte chunks addressed by lanes i/4, i/4+4, i/4+8, i/4+12.  Source lane s
  // therefore points at row key0 + s/4, channels dbase + 4*(s%4), and lane i ends up with
  // V[key0 + 0..3][dbase + i]: four consecutive keys of one channel, which is half of an
  // A-operand fragment of O^T += V^T P^T.
  unsigned char *vrd[2][2];   // [channel tile][which 4-key group]; add ks*2048 + buffer*8192
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);     // + 16*ks, which keeps (key>>1)&1
      const int off = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
      vrd[0][half] = vlds + off;
      vrd[1][half] = vlds + (off ^ 64);   // second channel tile: +64 bytes == flip of the swizzle bit
    }
  }
  const uint32_t lds_base =
      (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)vlds);

  // ---- the key tiles of the (clipped) 3x3 block neighbourhood, in raster order
  const int R0 = max(R - 1, 0), R1 = min(R + 1, p.nbh - 1);
  const int C0 = max(C - 1, 0), C1 = min(C + 1, p.nbw - 1);
  const int ncols = C1 - C0 + 1, ntiles = (R1 - R0 + 1) * ncols * TPB;
  auto key_tile_base = [&](int i) {
    const int sub = i & (TPB - 1), nbi = i / TPB;
    const int dR = (nbi >= ncols) + (nbi >= 2 * ncols);
    return (uint32_t)tile_base(R0 + dR, C0 + nbi - dR * ncols, sub) * rowB;
  };
  auto load_k = [&](bf16x8 (&kf)[2][4], uint32_t base) {
    const char *t = kb + base;
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int s = 0; s < 4; s++)
        kf[mt][s] = *reinterpret_cast<const bf16x8 *>(t + mt * kstep + koff + 16 * s);
  };
  auto dma_v = [&](int buf, uint32_t base) {
    const char *t = vb + base;
#pragma unroll
    for (int it = 0; it < 8; it++) dma16(t + vstep(it), voff, lds_base + buf * 8192 + it * 1024);
  };

  // ---- stage A: one 32x32 block of S^T
  auto stage_a = [&](const bf16x8 (&kf)[2][4], int mt, int nt) {
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qf[nt][ks], s, 0, 0, 0);
    return s;
  };
  // ---- stage C: O^T[:, nt] += V^T[:, keys of mt] P^T.  The accumulator layout of S^T (lane =
  // query column; register i = key 8*(i/4) + 4*hh + i%4) is the B-operand layout of this
  // product for the key order {4hh..4hh+3, 8+4hh..8+4hh+3} per 16 keys; the V fragments are
  // fetched in that same order.
  f32x16 o[2][2];   // [dt][nt]: channel rows 32*dt + 8*(i/4) + 4*hh + i%4, query column
  auto stage_c = [&](int mt, int nt, const bf16x8 (&pf)[2], int buf) {
#pragma unroll
    for (int sp = 0; sp < 2; sp++)
#pragma unroll
      for (int dt = 0; dt < 2; dt++) {
        const int off = buf * 8192 + (2 * mt + sp) * 2048;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][0] + off));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][1] + off));
        const bf16x4 lo4 = __builtin_bit_cast(bf16x4, lo), hi4 = __builtin_bit_cast(bf16x4, hi);
        const bf16x8 vf = {lo4[0], lo4[1], lo4[2], lo4[3], hi4[0], hi4[1], hi4[2], hi4[3]};
        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], o[dt][nt], 0, 0, 0);
      }
  };

  float m[2], l[2];
  // state initialised by the global token (key 0): m = its logit, l = 1, O = v_0
  auto init_state = [&]() {
    bf16x8 k0[4];
#pragma unroll
    for (int s = 0; s < 4; s++) k0[s] = *reinterpret_cast<const bf16x8 *>(kb + 64 * hh + 16 * s);
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
        const bf16x4 v4 = *reinterpret_cast<const bf16x4 *>(vb + (32 * dt + 8 * ig + 4 * hh) * 2);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[dt][0][4 * ig + e] = (float)v4[e];
          o[dt][1][4 * ig + e] = (float)v4[e];
        }
      }
  };

  bf16x8 kfa[2][4], kfb[2][4];

  // =========================== fast path: fixed exponent reference ===========================
  // the first key tile is requested before the state initialisation, so that its latency and
  // that of the global token's rows overlap
  dma_v(0, key_tile_base(0));
  load_k(kfa, key_tile_base(0));
  init_state();
  {
    float nm[2] = {-m[0], -m[1]};
    float la[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
    // stage B: element-wise weights of one 32x32 block
    auto stage_b = [&](const f32x16 &s, int nt, bf16x8 (&pf)[2]) {
#pragma unroll
      for (int i = 0; i < 16; i += 2) {
        const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i], p.c, nm[nt]));
        const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[i + 1], p.c, nm[nt]));
        la[nt][0] += p0;
        la[nt][1] += p1;
        const bf16x2 pk = __builtin_bit_cast(bf16x2, pack_bf16(p0, p1));
        pf[i >> 3][i & 7] = pk[0];
        pf[i >> 3][(i & 7) + 1] = pk[1];
      }
    };
    // One key tile.  Requests for the next tile go out first: V (into the other LDS buffer,
    // free since the previous tile finished), then K (into the other register set).  Loads
    // complete in issue order, so once the next tile's K registers are usable its V is in LDS.
    auto fast_tile = [&](int i, const bf16x8 (&kc)[2][4], bf16x8 (&kn)[2][4], int buf, f32x16 &s00) {
      const uint32_t nbase = key_tile_base(min(i + 1, ntiles - 1));
      dma_v(1 - buf, nbase);
      load_k(kn, nbase);
      bf16x8 p0[2], p1[2], p2[2], p3[2];
      const f32x16 s01 = stage_a(kc, 0, 1);
      stage_b(s00, 0, p0);
      const f32x16 s10 = stage_a(kc, 1, 0);
      stage_b(s01, 1, p1);
      stage_c(0, 0, p0, buf);
      const f32x16 s11 = stage_a(kc, 1, 1);
      stage_b(s10, 0, p2);
      stage_c(0, 1, p1, buf);
      s00 = stage_a(kn, 0, 0);            // first block of the next tile
      stage_b(s11, 1, p3);
      stage_c(1, 0, p2, buf);
      stage_c(1, 1, p3, buf);
    };
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // first tile: V and K both landed
    f32x16 s00 = stage_a(kfa, 0, 0);
    for (int i = 0; i < ntiles; i += 2) {
      fast_tile(i, kfa, kfb, 0, s00);
      if (i + 1 >= ntiles) break;
      fast_tile(i + 1, kfb, kfa, 1, s00);
    }
    l[0] += la[0][0] + la[0][1];
    l[1] += la[1][0] + la[1][1];
  }

  // the fast path is exact unless a weight overflowed: then some sum or output is not finite
  float big = fmaxf(fabsf(l[0]), fabsf(l[1]));
#pragma unroll
  for (int i = 0; i < 16; i++)
    big = fmaxf(fmaxf(big, fmaxf(fabsf(o[0][0][i]), fabsf(o[0][1][i]))),
                fmaxf(fabsf(o[1][0][i]), fabsf(o[1][1][i])));
  if (__any(!(big < 1e30f))) {
    // ====================== careful path: running maximum, tile by tile ======================
    init_state();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    for (int i = 0; i < ntiles; i++) {
      const uint32_t base = key_tile_base(i);
      dma_v(0, base);
      load_k(kfa, base);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
      for (int nt = 0; nt < 2; nt++) {
        const f32x16 s0 = stage_a(kfa, 0, nt), s1 = stage_a(kfa, 1, nt);
        float mx0 = fmaxf(s0[0], s0[1]), mx1 = fmaxf(s1[0], s1[1]);
#pragma unroll
        for (int e = 2; e < 16; e += 2) {
          mx0 = fmaxf(fmaxf(mx0, s0[e]), s0[e + 1]);
          mx1 = fmaxf(fmaxf(mx1, s1[e]), s1[e + 1]);
        }
        const float m_new = fmaxf(m[nt], half_swap_max(fmaxf(mx0, mx1)) * p.c);
        const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
        m[nt] = m_new;
        const float nm = -m_new;
        float ls = 0.f;
        bf16x8 pa[2], pb[2];
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
          const float a0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e], p.c, nm));
          const float a1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e + 1], p.c, nm));
          const float b0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e], p.c, nm));
          const float b1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e + 1], p.c, nm));
          ls += (a0 + a1) + (b0 + b1);
          const bf16x2 ka = __builtin_bit_cast(bf16x2, pack_bf16(a0, a1));
          const bf16x2 kb2 = __builtin_bit_cast(bf16x2, pack_bf16(b0, b1));
          pa[e >> 3][e & 7] = ka[0];
          pa[e >> 3][(e & 7) + 1] = ka[1];
          pb[e >> 3][e & 7] = kb2[0];
          pb[e >> 3][(e & 7) + 1] = kb2[1];
        }
        l[nt] = __builtin_fmaf(l[nt], alpha, ls);
#pragma unroll
        for (int e = 0; e < 16; e++) { o[0][nt][e] *= alpha; o[1][nt][e] *= alpha; }
        stage_c(0, nt, pa, 0);
        stage_c(1, nt, pb, 0);
      }
      asm volatile("" ::: "memory");   // the tile's LDS reads stay ahead of the next tile's transfer
    }
  }

  // ---- normalise and store: lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3
  char *ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const float inv = 1.f / half_swap_sum(l[nt]);
    char *row = ob + (size_t)(qbase + tile_off(l32 + 32 * nt)) * (size_t)(p.ost * 2) + 8 * hh;
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        uint2 u = {pack_bf16(o[dt][nt][4 * ig] * inv, o[dt][nt][4 * ig + 1] * inv),
                   pack_bf16(o[dt][nt][4 * ig + 2] * inv, o[dt][nt][4 * ig + 3] * inv)};
        *reinterpret_cast<uint2 *>(row + 64 * dt + 16 * ig) = u;
      }
  }
}

}  // namespace

bool mfma_attn_supported(const ns_attn_desc &d) {
  return d.dtype == NS_BF16 && d.head_dim == 64 && d.radius == 1 && d.n_global == 1 &&
         d.coords == nullptr && (d.block == 8 || d.block == 16) && d.grid_h % d.block == 0 &&
         d.grid_w % d.block == 0 && d.scale > 0.f &&
         // the kernel addresses tokens with 32-bit byte offsets from the (batch, head) base
         (long long)d.tokens * d.q_stride_t * 2 < 0x7fffffffLL &&
         (long long)d.tokens * d.out_stride_t * 2 < 0x7fffffffLL;
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
  const size_t lds = 4 * 16384;   // per wave: two V tiles
  if (d.block == 8)
    hipLaunchKernelGGL(attn_mfma_kernel<3>, dim3(p.total_wgs), dim3(256), lds, a.stream, p);
  else
    hipLaunchKernelGGL(attn_mfma_kernel<4>, dim3(p.total_wgs), dim3(256), lds, a.stream, p);
  return check_launch("attn_mfma_kernel");
}

}  // namespace ns
