// bf16 MFMA neighbourhood attention for blocks whose side is a multiple of 16: the four 64-query
// tiles of a 16x16 square share every key tile (gfx950).
//
// A 16x16 square is four tiles of 64 tokens (4 grid rows of 16), and all four have the same
// neighbourhood: the 16x16 squares of the (clipped) 3x3 blocks around the block the square lies
// in - up to 9 x 4 key tiles for 16x16 blocks, 36 x 4 for 32x32, 144 x 4 for 64x64.  A workgroup
// of 4 waves owns one square, wave w its tile w; the key tiles pass through a 3-slot LDS ring (direct
// global -> LDS transfers, a quarter of each issued by every wave, XOR-swizzled) and every wave
// uses every one of them: one fetch from L2 instead of four, and no wave ever idles.  One
// s_barrier per key tile makes the tile visible to all and frees the slot that the next transfer
// overwrites.  Mathematics, register formulation, fixed exponent reference and the redo of query
// tiles that overflow it are those of ns_attn_mfma.hip / ns_attn_sweep.hip.
#include "ns_common.h"

namespace ns {

namespace {

struct BlockParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float c;              // scale * log2(e)
  int grid_h, grid_w, nbh, nbw;   // 16x16 squares per side: ceil(grid / 16)
  int bm;               // squares per block side: block / 16
  int heads;
  int blocks;           // batch * heads * nbh * nbw
  int n_global;         // G leading global tokens, 1 .. 8 (their K and V rows sit in LDS)
};

typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
typedef bf16x8 __attribute__((address_space(3))) *lds_bf16x8_ptr;

constexpr uint32_t kSlot = 16384;     // one key tile: K [64][64] bf16, then V [64][64] bf16
constexpr uint32_t kVOff = 8192;
constexpr int kSlots = 3;
constexpr uint32_t kK0Row = 3 * 16384;         // k_0 in the first 128 bytes of a 1 KB transfer
constexpr uint32_t kV0Row = 3 * 16384 + 1024;  // v_0 likewise


#define NS_U(x) __builtin_amdgcn_readfirstlane(x)

constexpr float kMasked = -1e30f;     // logit of a key that does not exist (edge blocks of a grid 16 does not divide)

// grid: one workgroup of 256 threads per 16x16 square of queries.  EDGE: the grid has short squares
// at its right or bottom edge (a side that 16 does not divide).
template <bool EDGE>
__global__ __launch_bounds__(256, 2) void attn_block16_kernel(BlockParams p) {
  const int tid = threadIdx.x, wave = NS_U(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hh = lane >> 5;

  // consecutive blocks (raster order within an image) go to the same XCD: workgroups are dealt
  // round-robin to the 8 XCDs, and neighbouring query blocks share most of their key tiles
  int bid = blockIdx.x;
  if (p.blocks % 8 == 0) bid = (bid & 7) * (p.blocks / 8) + (bid >> 3);
  const int per_image = p.nbh * p.nbw;
  const int img = NS_U(bid / per_image), blk = bid - img * per_image;
  const int R = NS_U(blk / p.nbw), C = blk - R * p.nbw;
  const int b = NS_U(img / p.heads), h = img - b * p.heads;
  const char *qb = reinterpret_cast<const char *>(p.q + b * p.qsb + h * p.qsh);
  const char *kb = reinterpret_cast<const char *>(p.k + b * p.qsb + h * p.qsh);
  const char *vb = reinterpret_cast<const char *>(p.v + b * p.qsb + h * p.qsh);
  char *ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds_base = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);

  const uint32_t rowB = (uint32_t)p.qst * 2u;
  const uint32_t gridrowB = (uint32_t)p.grid_w * rowB;
  // tile `sub` of block (Rb, Cb) is grid rows 16*Rb + 4*sub .. +3, columns 16*Cb .. +15; its row i
  // is the token at grid row offset i/16, column offset i%16
  auto tile_token = [&](int Rb, int Cb, int sub) { return p.n_global + (Rb * 16 + sub * 4) * p.grid_w + Cb * 16; };
  // Short edge blocks: a tile is filled up with copies of existing tokens (row and column index
  // within the block are clamped).  A copied QUERY computes what its original computes and is
  // stored to the same place (same bits); a copied KEY gets the logit kMasked, i.e. the weight 0.
  const int hv_last = EDGE ? p.grid_h - 16 * (p.nbh - 1) : 16, wv_last = EDGE ? p.grid_w - 16 * (p.nbw - 1) : 16;
  auto rows_of = [&](int Rb) { return EDGE && Rb == p.nbh - 1 ? hv_last : 16; };
  auto cols_of = [&](int Cb) { return EDGE && Cb == p.nbw - 1 ? wv_last : 16; };
  // key tiles of a square that hold rows of their own (the others would be copies only: left out)
  const int subs_last = EDGE ? (hv_last + 3) >> 2 : 4;
  auto subs_of = [&](int Rb) { return EDGE && Rb == p.nbh - 1 ? subs_last : 4; };
  // offset of row i of tile `sub` of a block with hv rows and wv columns, from the tile's first token
  auto tile_off = [&](int i, int sub, int hv, int wv) {
    const int r = min(4 * sub + (i >> 4), hv - 1) - 4 * sub;      // may be negative: a tile without rows of its own
    return (uint32_t)(r * p.grid_w + min(i & 15, wv - 1)) * rowB;
  };
  // logits of keys that do not exist: accumulator register e (key half mt) of tile `sub` is block
  // row 4*sub + 2*mt + e/8 and column 8*((e/4)%2) + 4*hh + e%4
  auto mask_keys = [&](f32x16 &sv, int mt, int sub, int hv, int wv) {
#pragma unroll
    for (int e = 0; e < 16; e++)
      sv[e] = (4 * sub + 2 * mt + (e >> 3) >= hv || 8 * ((e >> 2) & 1) + 4 * hh + (e & 3) >= wv) ? kMasked : sv[e];
  };

  // ---- per-lane constants
  // transfers: request `it` of a tile is its rows 8*it .. 8*it+7 (half a grid row); LDS slot `lane`
  // holds row it*8 + lane/8, physical 16-byte chunk lane%8, which is logical chunk
  // (lane%8) ^ ((row>>1)&7) for K and (lane%8) ^ 4*((row>>1)&1) for V.  This wave issues requests
  // 2*wave and 2*wave+1 (grid row `wave` of the tile) of K and of V.
  const int drow = lane >> 3;
  const uint32_t dma_koff[2] = {drow * rowB + 16u * ((lane & 7) ^ ((drow >> 1) & 7)),
                                drow * rowB + 16u * ((lane & 7) ^ ((4 + (drow >> 1)) & 7))};
  const uint32_t dma_voff = drow * rowB + 16u * ((lane & 7) ^ (((drow >> 1) & 1) << 2));
  uint32_t krd[4];
#pragma unroll
  for (int s = 0; s < 4; s++) krd[s] = l32 * 128 + 16 * ((4 * hh + s) ^ ((l32 >> 1) & 7));
  uint32_t vrd[2][2];
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);
      const int off = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
      vrd[0][half] = kVOff + off;
      vrd[1][half] = kVOff + (off ^ 64);
    }
  }
  const uint32_t qoff0 = tile_off(l32, wave, rows_of(R), cols_of(C)) + 64u * hh;
  const uint32_t qoff1 = tile_off(l32 + 32, wave, rows_of(R), cols_of(C)) + 64u * hh;

  // ---- the key tiles of the (clipped) 3x3 block neighbourhood, square by square, four tiles each
  const int RB = NS_U(R / p.bm), CB = NS_U(C / p.bm);             // the block this square lies in
  const int R0 = max(RB - 1, 0) * p.bm, R1 = min((RB + 2) * p.bm, p.nbh) - 1;
  const int C0 = max(CB - 1, 0) * p.bm, C1 = min((CB + 2) * p.bm, p.nbw) - 1;
  const int ncb = C1 - C0 + 1, steps = ((R1 - R0) * 4 + subs_of(R1)) * ncb;
  int ir = R0, ic = C0, isub = 0, islot = 0;   // the tile to request next and its ring slot
  auto issue_next = [&]() {                    // this wave's share (4 requests); past the last tile it repeats that one
    // grid row `wave` of the tile (clamped to the block's last row), columns 8*j + lane/8 (clamped)
    const int grow = EDGE ? min(4 * isub + wave, rows_of(ir) - 1) : 4 * isub + wave;
    const uint32_t base = (uint32_t)tile_token(ir, ic, 0) * rowB + (uint32_t)grow * gridrowB;
    const uint32_t dst = lds_base + (uint32_t)islot * kSlot + (uint32_t)wave * 2048u;
    if (EDGE && ic == p.nbw - 1 && wv_last < 16) {
      // The lane offset of a transfer is unsigned, so the whole (clamped) column goes into it:
      // column min(8*j + lane/8, wv_last - 1) instead of 8*j in the base and lane/8 in the offset.
#pragma unroll
      for (int j = 0; j < 2; j++) {
        const uint32_t shift = (uint32_t)(min(8 * j + drow, wv_last - 1) - drow) * rowB;   // sum below is >= 0
        dma16(kb + base, dma_koff[j] + shift, dst + j * 1024);
        dma16(vb + base, dma_voff + shift, dst + kVOff + j * 1024);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 2; j++) dma16(kb + base + (size_t)j * 8 * rowB, dma_koff[j], dst + j * 1024);
#pragma unroll
      for (int j = 0; j < 2; j++) dma16(vb + base + (size_t)j * 8 * rowB, dma_voff, dst + kVOff + j * 1024);
    }
    islot = islot == kSlots - 1 ? 0 : islot + 1;
    const bool next_block = isub == subs_of(ir) - 1, next_row = next_block && ic == C1;
    const bool last = ir == R1 && next_row;
    isub = last ? isub : (next_block ? 0 : isub + 1);
    ic = last ? ic : (next_row ? C0 : (next_block ? ic + 1 : ic));
    ir = last ? ir : (next_row ? ir + 1 : ir);
  };

  // ---- register state of this wave's query tile
  bf16x8 qf[2][4];
  f32x16 o[2][2];
  float m[2], l[2], nm[2], la[2][2];

  auto stage_a = [&](const bf16x8 (&kf)[4], int nt) {
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[nt][ks], s, 0, 0, 0);
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
  // O^T[:, nt] += V^T[:, keys 32*mt ..] P^T; slot: byte offset of the key tile's ring slot
  auto stage_c = [&](int mt, int nt, const bf16x8 (&pf)[2], uint32_t slot) {
#pragma unroll
    for (int sp = 0; sp < 2; sp++)
#pragma unroll
      for (int dt = 0; dt < 2; dt++) {
        const uint32_t off = slot + (2 * mt + sp) * 2048;
        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smem + vrd[dt][0] + off));
        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smem + vrd[dt][1] + off));
        const bf16x4 a = __builtin_bit_cast(bf16x4, lo4), b2 = __builtin_bit_cast(bf16x4, hi4);
        const bf16x8 vf = {a[0], a[1], a[2], a[3], b2[0], b2[1], b2[2], b2[3]};
        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], o[dt][nt], 0, 0, 0);
      }
  };
  const char *qtile = qb + (uint32_t)tile_token(R, C, wave) * rowB;
  auto load_tile = [&]() {
#pragma unroll
    for (int s = 0; s < 4; s++) {
      qf[0][s] = *reinterpret_cast<const bf16x8 *>(qtile + (int32_t)qoff0 + 16 * s);
      qf[1][s] = *reinterpret_cast<const bf16x8 *>(qtile + (int32_t)qoff1 + 16 * s);
    }
  };
  // The state the global token gives a query tile: m = its logit (the fixed exponent reference),
  // l = 1, O = v_0; k_0 and v_0 sit in LDS.  The k_0 fragment is that of a key tile whose rows
  // are all k_0, so every register of its product with Q is q . k_0.  Further global tokens
  // (rows 1 .. G-1 of the same LDS areas) are added one by one with a running maximum, so the
  // reference becomes the largest of the global tokens' logits.
  auto init_tile = [&]() {
    bf16x8 k0[4];
#pragma unroll
    for (int s = 0; s < 4; s++) k0[s] = *(lds_bf16x8_ptr)(smem + kK0Row + 64 * hh + 16 * s);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const f32x16 s = stage_a(k0, nt);
      m[nt] = s[0] * p.c;
      nm[nt] = -m[nt];
      l[nt] = hh == 0 ? 1.f : 0.f;
      la[nt][0] = 0.f; la[nt][1] = 0.f;
    }
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++) {
        const u32x2 v2 = *(u32x2 __attribute__((address_space(3))) *)(smem + kV0Row + 64 * dt + 16 * ig + 8 * hh);
        const bf16x4 v4 = __builtin_bit_cast(bf16x4, v2);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[dt][0][4 * ig + e] = (float)v4[e];
          o[dt][1][4 * ig + e] = (float)v4[e];
        }
      }
    for (int g = 1; g < p.n_global; g++) {
      bf16x8 kg[4];
#pragma unroll
      for (int s = 0; s < 4; s++) kg[s] = *(lds_bf16x8_ptr)(smem + kK0Row + 128 * g + 64 * hh + 16 * s);
      float pg[2];
#pragma unroll
      for (int nt = 0; nt < 2; nt++) {
        const f32x16 s = stage_a(kg, nt);
        const float sg = s[0] * p.c, m_new = fmaxf(m[nt], sg);
        const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
        pg[nt] = __builtin_amdgcn_exp2f(sg - m_new);
        m[nt] = m_new;
        nm[nt] = -m_new;
        l[nt] = __builtin_fmaf(l[nt], alpha, hh == 0 ? pg[nt] : 0.f);
#pragma unroll
        for (int e = 0; e < 16; e++) { o[0][nt][e] *= alpha; o[1][nt][e] *= alpha; }
      }
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int ig = 0; ig < 4; ig++) {
          const u32x2 v2 = *(u32x2 __attribute__((address_space(3))) *)(smem + kV0Row + 128 * g + 64 * dt + 16 * ig + 8 * hh);
          const bf16x4 v4 = __builtin_bit_cast(bf16x4, v2);
#pragma unroll
          for (int e = 0; e < 4; e++) {
            o[dt][0][4 * ig + e] = __builtin_fmaf(pg[0], (float)v4[e], o[dt][0][4 * ig + e]);
            o[dt][1][4 * ig + e] = __builtin_fmaf(pg[1], (float)v4[e], o[dt][1][4 * ig + e]);
          }
        }
    }
  };
  // normalise and store; returns whether a weight overflowed the fixed reference (then some sum or
  // output is not finite).  Lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3.
  auto finish_tile = [&]() {
    l[0] += la[0][0] + la[0][1];
    l[1] += la[1][0] + la[1][1];
    float big = fmaxf(fabsf(l[0]), fabsf(l[1]));
#pragma unroll
    for (int i = 0; i < 16; i++)
      big = fmaxf(fmaxf(big, fmaxf(fabsf(o[0][0][i]), fabsf(o[0][1][i]))),
                  fmaxf(fabsf(o[1][0][i]), fabsf(o[1][1][i])));
    const bool bad = __any(!(big < 1e30f));
    char *t = ob + (size_t)tile_token(R, C, wave) * (size_t)(p.ost * 2);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const float inv = 1.f / half_swap_sum(l[nt]);
      const int i = l32 + 32 * nt;
      const int r = min(4 * wave + (i >> 4), rows_of(R) - 1) - 4 * wave;   // as in tile_off
      char *row = t + (ptrdiff_t)(r * p.grid_w + min(i & 15, cols_of(C) - 1)) * (ptrdiff_t)(p.ost * 2) + 8 * hh;
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int ig = 0; ig < 4; ig++) {
          const u32x2 u = {pack_bf16(o[dt][nt][4 * ig] * inv, o[dt][nt][4 * ig + 1] * inv),
                           pack_bf16(o[dt][nt][4 * ig + 2] * inv, o[dt][nt][4 * ig + 3] * inv)};
          *reinterpret_cast<u32x2 *>(row + 64 * dt + 16 * ig) = u;
        }
    }
    return bad;
  };

  // ---- prologue: the first three key tiles are requested, the first has landed
  if (wave == 0) {
    // the global tokens' rows, 8 lanes x 16 bytes each: LDS row r = token min(r, G-1)
    const uint32_t goff = (uint32_t)min(lane >> 3, p.n_global - 1) * rowB + 16u * (lane & 7);
    dma16(kb, goff, lds_base + kK0Row);
    dma16(vb, goff, lds_base + kV0Row);
  }
  issue_next();
  issue_next();
  issue_next();
  wait_vm<8>();                     // k_0, v_0 and tile 0
  __syncthreads();
  load_tile();                       // consumed at once: no load is pending at the loop head
  init_tile();

  int cslot = 0;
  int cr = R0, cc = C0, csub = 0;      // the key tile in work
  for (int s = 0; s < steps; s++) {
    const uint32_t slot = (uint32_t)cslot * kSlot;
    const int hvk = rows_of(cr), wvk = cols_of(cc);
    const bool edge = EDGE && (hvk < 4 * csub + 4 || wvk < 16);
    {
      bf16x8 kA[4], kB[4], p0[2], p1[2], p2[2], p3[2];
#pragma unroll
      for (int t = 0; t < 4; t++) {
        kA[t] = *(lds_bf16x8_ptr)(smem + slot + krd[t]);
        kB[t] = *(lds_bf16x8_ptr)(smem + slot + 4096 + krd[t]);
      }
      f32x16 s00 = stage_a(kA, 0);
      if (edge) mask_keys(s00, 0, csub, hvk, wvk);
      f32x16 s01 = stage_a(kA, 1);
      if (edge) mask_keys(s01, 0, csub, hvk, wvk);
      stage_b(s00, 0, p0);
      f32x16 s10 = stage_a(kB, 0);
      if (edge) mask_keys(s10, 1, csub, hvk, wvk);
      stage_b(s01, 1, p1);
      stage_c(0, 0, p0, slot);
      f32x16 s11 = stage_a(kB, 1);
      if (edge) mask_keys(s11, 1, csub, hvk, wvk);
      stage_b(s10, 0, p2);
      stage_c(0, 1, p1, slot);
      stage_b(s11, 1, p3);
      stage_c(1, 0, p2, slot);
      stage_c(1, 1, p3, slot);
    }
    wait_vm<4>();     // tile s+1: this wave's share has landed (its share of tile s+2 may still be in flight)
    __syncthreads();   // ... and everybody's; and everybody is done with tile s, whose slot tile s+3 takes
    issue_next();
    cslot = cslot == kSlots - 1 ? 0 : cslot + 1;
    if (EDGE) {        // the same order as the requests
      const bool nb2 = csub == subs_of(cr) - 1, nr2 = nb2 && cc == C1;
      csub = nb2 ? 0 : csub + 1;
      cc = nr2 ? C0 : (nb2 ? cc + 1 : cc);
      cr = nr2 ? cr + 1 : cr;
    }
  }
  wait_vm<0>();
  const bool bad = finish_tile();
  __syncthreads();                   // the ring is free: each wave takes 16 KB of it below
  if (!bad) return;

  // ---- a weight overflowed in this wave's query tile (its stored rows are not finite): once
  // more with a running maximum, fragments straight from global memory, V staged through LDS
  const uint32_t mine = (uint32_t)wave * 16384u;
  load_tile();
  init_tile();
  for (int rr = R0; rr <= R1; rr++)
    for (int cc2 = C0; cc2 <= C1; cc2++)
      for (int sub = 0; sub < subs_of(rr); sub++) {
        const int cc = cc2;
        const char *kbase = kb + (uint32_t)tile_token(rr, cc, sub) * rowB;
        const uint32_t vblock = (uint32_t)tile_token(rr, cc, 0) * rowB;
        const int hvk = rows_of(rr), wvk = cols_of(cc);
        bf16x8 kt[2][4];
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
#pragma unroll
          for (int t = 0; t < 4; t++)
            kt[mt][t] = *reinterpret_cast<const bf16x8 *>(kbase + (int32_t)tile_off(l32 + 32 * mt, sub, hvk, wvk) + 64 * hh + 16 * t);
#pragma unroll
        for (int it = 0; it < 8; it++) {
          const int grow = min(4 * sub + (it >> 1), hvk - 1);
          // (unsigned lane offset: the clamped column goes into it whole, see issue_next)
          const uint32_t shift = (uint32_t)(min(8 * (it & 1) + drow, wvk - 1) - drow) * rowB;
          dma16(vb + vblock + (size_t)grow * gridrowB, dma_voff + shift, lds_base + mine + kVOff + it * 1024);
        }
        wait_vm<0>();               // also the K fragments above
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
          f32x16 s0 = stage_a(kt[0], nt), s1 = stage_a(kt[1], nt);
          if (EDGE && (hvk < 4 * sub + 4 || wvk < 16)) {
            mask_keys(s0, 0, sub, hvk, wvk);
            mask_keys(s1, 1, sub, hvk, wvk);
          }
          float mx0 = fmaxf(s0[0], s0[1]), mx1 = fmaxf(s1[0], s1[1]);
#pragma unroll
          for (int e = 2; e < 16; e += 2) {
            mx0 = fmaxf(fmaxf(mx0, s0[e]), s0[e + 1]);
            mx1 = fmaxf(fmaxf(mx1, s1[e]), s1[e + 1]);
          }
          const float m_new = fmaxf(m[nt], half_swap_max(fmaxf(mx0, mx1)) * p.c);
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
          stage_c(0, nt, pa, mine);
          stage_c(1, nt, pb, mine);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // V reads done before the next transfer into the slot
      }
  finish_tile();
}

}  // namespace

bool block16_attn_supported(const ns_attn_desc &d) {
  return d.dtype == NS_BF16 && d.head_dim == 64 && d.radius == 1 && d.n_global >= 1 && d.n_global <= 8 &&
         d.coords == nullptr && d.block >= 16 && d.block % 16 == 0 && d.scale > 0.f &&
         // tokens are addressed with 32-bit byte offsets from the (batch, head) base
         (long long)d.tokens * d.q_stride_t * 2 < 0x7fffffffLL &&
         (long long)d.tokens * d.out_stride_t * 2 < 0x7fffffffLL;
}

ns_status launch_attn_block16(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  BlockParams p;
  p.q = static_cast<const uint16_t *>(a.q);
  p.k = static_cast<const uint16_t *>(a.k);
  p.v = static_cast<const uint16_t *>(a.v);
  p.out = static_cast<uint16_t *>(a.out);
  p.qsb = d.q_stride_b; p.qsh = d.q_stride_h; p.qst = d.q_stride_t;
  p.osb = d.out_stride_b; p.osh = d.out_stride_h; p.ost = d.out_stride_t;
  p.c = d.scale * kLog2e;
  p.grid_h = d.grid_h;
  p.grid_w = d.grid_w;
  p.nbh = (d.grid_h + 15) / 16;
  p.nbw = (d.grid_w + 15) / 16;
  p.bm = d.block / 16;
  p.heads = d.heads;
  p.n_global = d.n_global;
  const long long blocks = (long long)d.batch * d.heads * p.nbh * p.nbw;
  if (blocks > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "launch grid too large");
  p.blocks = (int)blocks;
  const int lds = 4 * 16384;        // three ring slots and the global token's rows; the redo gives each wave a slot
  const bool even = d.grid_h % 16 == 0 && d.grid_w % 16 == 0;
  const ns_status rs = reserve_lds_once(even ? reinterpret_cast<const void *>(attn_block16_kernel<false>)
                                             : reinterpret_cast<const void *>(attn_block16_kernel<true>), lds);
  if (rs != NS_OK) return rs;
  if (d.grid_h % 16 == 0 && d.grid_w % 16 == 0)
    hipLaunchKernelGGL(attn_block16_kernel<false>, dim3((unsigned)blocks), dim3(256), lds, a.stream, p);
  else
    hipLaunchKernelGGL(attn_block16_kernel<true>, dim3((unsigned)blocks), dim3(256), lds, a.stream, p);
  return check_launch("attn_block16_kernel");
}

}  // namespace ns
