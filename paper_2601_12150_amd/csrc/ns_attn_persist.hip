// Persistent bf16 MFMA neighbourhood attention for patch queries on the full grid (gfx950).
// ALTERNATIVE kernel, selected with NSATTN_KERNEL=persist; the default is ns_attn_mfma.hip.  It is
// correct (same parity tests) and hides memory latency better, but at present loses what it gains
// to register moves between the vector and accumulator register files at the branches inside its
// tile body (first/last key tile of a query tile); the default kernel is faster until those
// branches are peeled into separate code paths.
//
// Same mathematics and register formulation as ns_attn_mfma.hip (transposed products, P kept in
// registers, fixed exponent reference with a checked fallback); what differs is how the chip is
// occupied.  One wave per SIMD (up to 512 VGPRs, 40 KB of LDS each) lives for the whole launch and
// walks a list of 64-query tiles.  All global traffic of the steady state is asynchronous and
// request-ordered:
//   K tile  global -> LDS (2-slot ring, coalesced 1 KB requests, XOR swizzle) -> registers one
//           tile ahead of its use,
//   V tile  global -> LDS (3-slot ring) -> ds_read_b64_tr_b16 at its use,
//   Q, k_0, v_0 of the NEXT query tile global -> registers (ordinary loads) while the current
//           one is computed.
// Requests run two key tiles ahead and do not stop at query-tile boundaries, so neither the
// per-query prologue nor any memory latency is exposed after the first tile of a wave.  The
// waits on the LDS transfers are explicit vmcnt(N): vector loads complete in issue order, so "at
// most N outstanding" means everything but the N youngest requests has arrived.  Extra requests
// in flight (stores, next-query loads) can only make such a wait conservative, never early; and
// the waits the compiler computes for its own loads are conservative for the same reason (it
// does not count the transfers).  Only requests WITHOUT a register result are issued from asm:
// a register written asynchronously by asm would look free to the register allocator.
#include "ns_common.h"

namespace ns {

namespace {

struct PersistParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float c;              // scale * log2(e)
  int grid_w, nbh, nbw;
  int heads;
  int tiles_per_image;  // 64-query tiles per (batch, head)
  int tiles_total;
  int num_wgs, xcds, slots;   // slots: waves per XCD
};

typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
typedef bf16x8 __attribute__((address_space(3))) *lds_bf16x8_ptr;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float hswap_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float hswap_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// 16 bytes per lane, global -> LDS at lds + 16*lane, no registers.
__device__ __forceinline__ void dma16(const char *base, uint32_t voff, uint32_t lds) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds), "v"(voff), "s"(base) : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int LOG2B>
__global__ __launch_bounds__(64) void attn_mfma_persist_kernel(PersistParams p) {
  constexpr int B_ = 1 << LOG2B;
  constexpr int TPB = (B_ * B_) / 64;
  constexpr int TROWS = 64 / B_;
  // one wave per workgroup: four of them share a CU (one per SIMD, by their register count), each
  // with its own 40 KB of LDS, so LDS addresses stay small and no workgroup-level state exists
  const int lane = threadIdx.x;
  const int l32 = lane & 31, hh = lane >> 5;

  // ---- this wave's query tiles: XCD x owns a contiguous range of the (image-major) tile list,
  // its waves sweep that range together (tile = lo + slot + j*slots), so the XCD's L2 holds one
  // or two head-images' K and V at a time
  // (integer division runs on the vector ALU; readfirstlane puts the uniform results back into
  // scalar registers so that everything derived from them stays scalar)
#define NS_U(x) __builtin_amdgcn_readfirstlane(x)
  const int xcd = NS_U((int)blockIdx.x % p.xcds), slot = NS_U((int)blockIdx.x / p.xcds);
  const int slots = p.slots;
  const int lo = NS_U((int)((long long)p.tiles_total * xcd / p.xcds));
  const int hi = NS_U((int)((long long)p.tiles_total * (xcd + 1) / p.xcds));
  const int qt = lo + slot;
  if (qt >= hi) return;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *wlds = smem;                 // [0,16K): K ring (2 slots), [16K,40K): V ring (3 slots)
  const uint32_t lds_base = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)wlds);
  constexpr uint32_t VRING = 16384;

  const uint32_t rowB = (uint32_t)p.qst * 2u;
  const uint32_t gridrowB = (uint32_t)p.grid_w * rowB;
  auto tile_off = [&](int i) { return (i >> LOG2B) * p.grid_w + (i & (B_ - 1)); };
  auto tile_base = [&](int R2, int C2, int sub) { return 1 + (R2 * B_ + sub * TROWS) * p.grid_w + C2 * B_; };

  // ---- per-lane constants
  // DMA source: LDS slot `lane` of chunk `it` holds row it*8 + lane/8, physical 16-byte chunk lane%8.
  // K: logical chunk = physical ^ ((row>>1)&7); V: logical = physical ^ 4*((row>>1)&1).
  // For V, (row>>1)&1 does not depend on `it`; for K, (row>>1)&7 = (4*(it&1) + (row%8 >> 1)) & 7, so
  // even and odd requests use one offset register each.
  const int drow = lane >> 3;
  const uint32_t dma_koff[2] = {
      (uint32_t)tile_off(drow) * rowB + 16u * ((lane & 7) ^ ((drow >> 1) & 7)),
      (uint32_t)tile_off(drow) * rowB + 16u * ((lane & 7) ^ ((4 + (drow >> 1)) & 7))};
  const uint32_t dma_voff = (uint32_t)tile_off(drow) * rowB + 16u * ((lane & 7) ^ (((drow >> 1) & 1) << 2));
  auto dstep = [&](int it) { return LOG2B == 3 ? it * gridrowB : (it >> 1) * gridrowB + (it & 1) * 8u * rowB; };
  // K fragment reads: lane (row l32 [+32], half hh) needs logical chunks 4*hh + s
  unsigned char *krd[4];
#pragma unroll
  for (int s = 0; s < 4; s++) krd[s] = wlds + l32 * 128 + 16 * ((4 * hh + s) ^ ((l32 >> 1) & 7));
  // V transposed reads (see ns_attn_mfma.hip for the layout argument)
  unsigned char *vrd[2][2];
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);
      const int off = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
      vrd[0][half] = wlds + VRING + off;
      vrd[1][half] = wlds + VRING + (off ^ 64);
    }
  }
  const uint32_t qoff0 = (uint32_t)tile_off(l32) * rowB + 64u * hh;
  const uint32_t qoff1 = (uint32_t)tile_off(l32 + 32) * rowB + 64u * hh;

  // ---- cursors over this wave's flattened (query tile, key tile) sequence
  struct Cursor {
    int qt;                  // query tile id; clamped to the wave's last one
    int i, ntiles;           // key tile index within the query tile
    int R0, C0, ncols, R, C, qsub;
    const char *qb, *kb, *vb;
    char *ob;
  };
  auto open_query = [&](Cursor &c, int t) {
    c.qt = t;
    const int img = NS_U(t / p.tiles_per_image), rem = t - img * p.tiles_per_image;
    const int b = NS_U(img / p.heads), h = img - b * p.heads;
    const int blk = rem / TPB;               // TPB is a power of two
    c.qsub = rem % TPB;
    c.R = NS_U(blk / p.nbw); c.C = blk - c.R * p.nbw;
    c.R0 = max(c.R - 1, 0); c.C0 = max(c.C - 1, 0);
    const int R1 = min(c.R + 1, p.nbh - 1), C1 = min(c.C + 1, p.nbw - 1);
    c.ncols = C1 - c.C0 + 1;
    c.ntiles = (R1 - c.R0 + 1) * c.ncols * TPB;
    c.i = 0;
    const int64_t ho = b * p.qsb + h * p.qsh;
    c.qb = reinterpret_cast<const char *>(p.q + ho);
    c.kb = reinterpret_cast<const char *>(p.k + ho);
    c.vb = reinterpret_cast<const char *>(p.v + ho);
    c.ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);
  };
  auto key_base = [&](const Cursor &c) {
    const int sub = c.i & (TPB - 1), nbi = c.i / TPB;
    const int dR = (nbi >= c.ncols) + (nbi >= 2 * c.ncols);
    return (uint32_t)tile_base(c.R0 + dR, c.C0 + nbi - dR * c.ncols, sub) * rowB;
  };
  // next key tile; past the wave's last key tile the cursor stays on it (requests repeat, harmless)
  auto advance = [&](Cursor &c) {
    if (c.i + 1 < c.ntiles) { c.i++; return; }
    if (c.qt + slots < hi) open_query(c, c.qt + slots);
  };
  auto dma_k = [&](const Cursor &c, int slot) {
    const char *t = c.kb + key_base(c);
#pragma unroll
    for (int it = 0; it < 8; it++) dma16(t + dstep(it), dma_koff[it & 1], lds_base + slot * 8192 + it * 1024);
  };
  auto dma_v = [&](const Cursor &c, int slot) {
    const char *t = c.vb + key_base(c);
#pragma unroll
    for (int it = 0; it < 8; it++) dma16(t + dstep(it), dma_voff, lds_base + VRING + slot * 8192 + it * 1024);
  };

  // ---- register state
  bf16x8 qf[2][4], qn[2][4];       // Q fragments of the current / next query tile
  bf16x8 k0n[4];                   // k_0 slice and v_0 slice of the next query tile's image
  u32x2 v0n[2][4];
  bf16x8 kfa[2][4], kfb[2][4];     // K fragments, alternating by key tile parity
  f32x16 o[2][2];
  float m[2], l[2], nm[2], la[2][2];

  auto load_query = [&](const Cursor &c, bf16x8 (&qd)[2][4]) {
    const char *t = c.qb + (uint32_t)tile_base(c.R, c.C, c.qsub) * rowB;
#pragma unroll
    for (int s = 0; s < 4; s++) {
      qd[0][s] = *reinterpret_cast<const bf16x8 *>(t + qoff0 + 16 * s);
      qd[1][s] = *reinterpret_cast<const bf16x8 *>(t + qoff1 + 16 * s);
      k0n[s] = *reinterpret_cast<const bf16x8 *>(c.kb + 64 * hh + 16 * s);
    }
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++)
        v0n[dt][ig] = *reinterpret_cast<const u32x2 *>(c.vb + 8 * hh + 64 * dt + 16 * ig);
  };
  // the global token initialises the state: m = its logit (the fixed exponent reference),
  // l = 1, O = v_0.  Uses qf (already the new query's) and k0n / v0n.
  auto init_state = [&]() {
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      float acc = 0.f;
#pragma unroll
      for (int s = 0; s < 4; s++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc = __builtin_fmaf((float)qf[nt][s][j], (float)k0n[s][j], acc);
      acc = hswap_sum(acc);
      m[nt] = acc * p.c;
      nm[nt] = -m[nt];
      l[nt] = hh == 0 ? 1.f : 0.f;
      la[nt][0] = 0.f; la[nt][1] = 0.f;
    }
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        const bf16x4 v4 = __builtin_bit_cast(bf16x4, v0n[dt][ig]);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[dt][0][4 * ig + e] = (float)v4[e];
          o[dt][1][4 * ig + e] = (float)v4[e];
        }
      }
  };
  auto read_kf = [&](bf16x8 (&kf)[2][4], int slot) {
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int s = 0; s < 4; s++)
        kf[mt][s] = *(lds_bf16x8_ptr)(krd[s] + slot * 8192 + mt * 4096);
  };
  auto stage_a = [&](const bf16x8 (&kf)[2][4], const bf16x8 (&qq)[2][4], int mt, int nt) {
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qq[nt][ks], s, 0, 0, 0);
    return s;
  };
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
  auto stage_c = [&](int mt, int nt, const bf16x8 (&pf)[2], uint32_t voffs) {
#pragma unroll
    for (int sp = 0; sp < 2; sp++)
#pragma unroll
      for (int dt = 0; dt < 2; dt++) {
        const uint32_t off = voffs + (2 * mt + sp) * 2048;
        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][0] + off));
        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][1] + off));
        const bf16x4 a = __builtin_bit_cast(bf16x4, lo4), b2 = __builtin_bit_cast(bf16x4, hi4);
        const bf16x8 vf = {a[0], a[1], a[2], a[3], b2[0], b2[1], b2[2], b2[3]};
        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], o[dt][nt], 0, 0, 0);
      }
  };

  Cursor cc, pc;                   // consumer, producer (two key tiles ahead)
  open_query(cc, qt);
  open_query(pc, qt);

  // ---- prologue: the only place where this wave waits for a full round trip
  load_query(cc, qf);
  dma_k(pc, 0); dma_v(pc, 0); advance(pc);
  dma_k(pc, 1); dma_v(pc, 1); advance(pc);
  wait_vm<0>();
  init_state();
  read_kf(kfa, 0);
  f32x16 s00 = stage_a(kfa, qf, 0, 0);
  bf16x8 p3[2];                    // weights of the previous tile's last sub-block (deferred stage C)
  uint32_t vprev = 0;

  int vslot = 0;                   // V ring slot of the current key tile
  bool have_next_q = false;

  // One key tile.  kc: this tile's K fragments, kn: register set for the next tile's, kslot: K ring
  // slot of this tile (the next tile's is 1 - kslot).
  auto tile = [&](const bf16x8 (&kc)[2][4], bf16x8 (&kn)[2][4], int kslot, bool &done) {
    const bool first = cc.i == 0, last = cc.i + 1 == cc.ntiles;
    const uint32_t vcur = vslot * 8192u;
    // K of the tile after next goes into this tile's ring slot (its fragments are in registers)
    dma_k(pc, kslot);
    if (first) {
      // next query tile's Q, k_0, v_0: requested a whole query tile ahead
      Cursor nq = cc;
      have_next_q = cc.qt + slots < hi;
      if (have_next_q) { open_query(nq, cc.qt + slots); load_query(nq, qn); }
    }
    bf16x8 p0[2], p1[2], p2[2];
    // step 0
    const f32x16 s01 = stage_a(kc, qf, 0, 1);
    stage_b(s00, 0, p0);
    if (!first) stage_c(1, 1, p3, vprev);          // previous tile's last sub-block
    // V of the tile after next: its ring slot was last read just above
    dma_v(pc, vslot == 0 ? 2 : vslot - 1);
    advance(pc);
    // everything but the youngest requests (K, V of tile+2; V of tile+1 ...) has landed:
    // this tile's V and the next tile's K are in LDS
    wait_vm<24>();
    read_kf(kn, 1 - kslot);
    // step 1
    const f32x16 s10 = stage_a(kc, qf, 1, 0);
    stage_b(s01, 1, p1);
    stage_c(0, 0, p0, vcur);
    // step 2
    const f32x16 s11 = stage_a(kc, qf, 1, 1);
    stage_b(s10, 0, p2);
    stage_c(0, 1, p1, vcur);
    if (!last) {
      // step 3
      s00 = stage_a(kn, qf, 0, 0);
      stage_b(s11, 1, p3);
      stage_c(1, 0, p2, vcur);
      vprev = vcur;
    } else {
      // last key tile of this query tile: finish it, store, and switch to the next query tile
      stage_b(s11, 1, p3);
      stage_c(1, 0, p2, vcur);
      stage_c(1, 1, p3, vcur);
      l[0] += la[0][0] + la[0][1];
      l[1] += la[1][0] + la[1][1];
      float big = fmaxf(fabsf(l[0]), fabsf(l[1]));
#pragma unroll
      for (int i = 0; i < 16; i++)
        big = fmaxf(fmaxf(big, fmaxf(fabsf(o[0][0][i]), fabsf(o[0][1][i]))),
                    fmaxf(fabsf(o[1][0][i]), fabsf(o[1][1][i])));
      if (__any(!(big < 1e30f))) {
        // ---- a weight overflowed: redo this query tile with a running maximum.  Drain the
        // request pipeline first (the rings keep the data already requested for later tiles),
        // stage V through the ring slot this tile has just finished with.
        wait_vm<0>();
        // k0n / v0n hold the NEXT query's rows by now; keep them and reload this image's
        bf16x8 k0s[4];
        u32x2 v0s[2][4];
#pragma unroll
        for (int s = 0; s < 4; s++) {
          k0s[s] = k0n[s];
          k0n[s] = *reinterpret_cast<const bf16x8 *>(cc.kb + 64 * hh + 16 * s);
        }
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
          for (int ig = 0; ig < 4; ig++) {
            v0s[dt][ig] = v0n[dt][ig];
            v0n[dt][ig] = *reinterpret_cast<const u32x2 *>(cc.vb + 8 * hh + 64 * dt + 16 * ig);
          }
        init_state();
        Cursor rc = cc;
        for (rc.i = 0; rc.i < rc.ntiles; rc.i++) {
          const uint32_t base = key_base(rc);
          // K fragments straight from global memory (tracked loads: the pipeline is drained)
          bf16x8 kt[2][4];
          const char *t = rc.kb + base;
          const uint32_t kstep = (32 >> LOG2B) * gridrowB;
#pragma unroll
          for (int mt = 0; mt < 2; mt++)
#pragma unroll
            for (int s = 0; s < 4; s++)
              kt[mt][s] = *reinterpret_cast<const bf16x8 *>(t + mt * kstep + qoff0 + 16 * s);
          dma_v(rc, vslot);
          wait_vm<0>();
#pragma unroll
          for (int nt = 0; nt < 2; nt++) {
            const f32x16 s0 = stage_a(kt, qf, 0, nt), s1 = stage_a(kt, qf, 1, nt);
            float mx0 = fmaxf(s0[0], s0[1]), mx1 = fmaxf(s1[0], s1[1]);
#pragma unroll
            for (int e = 2; e < 16; e += 2) {
              mx0 = fmaxf(fmaxf(mx0, s0[e]), s0[e + 1]);
              mx1 = fmaxf(fmaxf(mx1, s1[e]), s1[e + 1]);
            }
            const float m_new = fmaxf(m[nt], hswap_max(fmaxf(mx0, mx1)) * p.c);
            const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
            m[nt] = m_new;
            const float nmm = -m_new;
            float ls = 0.f;
            bf16x8 pa[2], pb[2];
#pragma unroll
            for (int e = 0; e < 16; e += 2) {
              const float a0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e], p.c, nmm));
              const float a1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0[e + 1], p.c, nmm));
              const float b0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e], p.c, nmm));
              const float b1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1[e + 1], p.c, nmm));
              ls += (a0 + a1) + (b0 + b1);
              const bf16x2 ka = __builtin_bit_cast(bf16x2, pack_bf16(a0, a1));
              const bf16x2 kb2 = __builtin_bit_cast(bf16x2, pack_bf16(b0, b1));
              pa[e >> 3][e & 7] = ka[0]; pa[e >> 3][(e & 7) + 1] = ka[1];
              pb[e >> 3][e & 7] = kb2[0]; pb[e >> 3][(e & 7) + 1] = kb2[1];
            }
            l[nt] = __builtin_fmaf(l[nt], alpha, ls);
#pragma unroll
            for (int e = 0; e < 16; e++) { o[0][nt][e] *= alpha; o[1][nt][e] *= alpha; }
            stage_c(0, nt, pa, vcur);
            stage_c(1, nt, pb, vcur);
          }
          asm volatile("" ::: "memory");
        }
        // put the next query's rows back
#pragma unroll
        for (int s = 0; s < 4; s++) k0n[s] = k0s[s];
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
          for (int ig = 0; ig < 4; ig++) v0n[dt][ig] = v0s[dt][ig];
      }
      // ---- normalise and store: lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3
      {
        const int qbase = tile_base(cc.R, cc.C, cc.qsub);
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
          const float inv = 1.f / hswap_sum(l[nt]);
          char *row = cc.ob + (size_t)(qbase + tile_off(l32 + 32 * nt)) * (size_t)(p.ost * 2) + 8 * hh;
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
      if (!have_next_q) { done = true; return; }
      // ---- next query tile: its Q, k_0, v_0 were requested at this one's first key tile
#pragma unroll
      for (int nt = 0; nt < 2; nt++)
#pragma unroll
        for (int s = 0; s < 4; s++) qf[nt][s] = qn[nt][s];
      init_state();
      s00 = stage_a(kn, qf, 0, 0);
    }
    vslot = vslot == 2 ? 0 : vslot + 1;
    advance(cc);
  };

  bool done = false;
  while (true) {
    tile(kfa, kfb, 0, done);
    if (done) break;
    tile(kfb, kfa, 1, done);
    if (done) break;
  }
}

}  // namespace

bool persist_attn_supported(const ns_attn_desc &d) {
  return mfma_attn_supported(d);
}

ns_status launch_attn_persist(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  static int num_cus = 0;
  if (num_cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
      return fail(NS_ERR_HIP, "cannot query the device");
    num_cus = prop.multiProcessorCount;
  }
  PersistParams p;
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
  const long long tt = (long long)p.tiles_per_image * d.heads * d.batch;
  if (tt > 0x3fffffffLL) return fail(NS_ERR_UNSUPPORTED, "too many query tiles");
  p.tiles_total = (int)tt;
  p.xcds = (num_cus % 8 == 0) ? 8 : 1;
  p.num_wgs = num_cus * 4;                   // one single-wave workgroup per SIMD
  p.slots = p.num_wgs / p.xcds;
  const size_t lds = 40960;
  if (d.block == 8)
    hipLaunchKernelGGL(attn_mfma_persist_kernel<3>, dim3(p.num_wgs), dim3(64), lds, a.stream, p);
  else
    hipLaunchKernelGGL(attn_mfma_persist_kernel<4>, dim3(p.num_wgs), dim3(64), lds, a.stream, p);
  return check_launch("attn_mfma_persist_kernel");
}

}  // namespace ns
