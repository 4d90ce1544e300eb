// bf16 MFMA neighbourhood attention for patch queries over per-block token lists (gfx950): pruned
// sequences, grids that the block side does not divide, and block sides other than 8 and 16.
//
// After pruning (paper, "Time-Efficiency Optimization") the sequence is [CLS; surviving patches] and
// the mask is still evaluated on each survivor's original grid position (paper, "Memory-Efficiency
// Optimization").  block_lists_kernel has bucketed the
// survivors by block (grid_lists_kernel does the same for a complete grid whose last blocks may be
// short).  A block's list is cut into runs of 64 entries: a wave owns one run as its query tile
// and walks the runs of the up to nine neighbouring blocks as key tiles, the rows beyond a run's
// fill masked.
//
// Same register formulation as ns_attn_mfma.hip: S^T = K Q^T and O^T += V^T P^T with
// v_mfma_f32_32x32x16_bf16, P kept in registers, K fragments gathered straight from global memory
// (one row address per lane), V gathered global -> LDS with direct 16-byte transfers and read
// transposed with ds_read_b64_tr_b16.  The softmax keeps a running maximum per query (this
// kernel is not the tuned one: no fixed exponent reference, no sub-block pipeline); the next
// tile's K and V are requested as soon as the current tile's logits are computed.
#include "ns_common.h"

namespace ns {

namespace {

struct RaggedParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float c;               // scale * log2(e)
  int nbh, nbw, cap;     // blocks per side, slots per block in `lists`
  int tpb;               // runs of 64 slots per block: ceil(cap / 64)
  int n_global;          // leading global tokens (keys of every query)
  int heads;
  const int32_t *lists;  // [B, nbh*nbw, cap] token indices
  const int32_t *counts; // [B, nbh*nbw]
};

typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;


// grid (ceil(nblocks*tpb/4), H, B), 256 threads: one wave per query tile (tpb = runs per block).
__global__ __launch_bounds__(256, 2) void attn_mfma_ragged_kernel(RaggedParams p) {
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hh = lane >> 5;
  const int nblocks = p.nbh * p.nbw;
  // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous range of blocks, so
  // that the K and V rows which neighbouring blocks share are fetched into one L2 only
  int bx = blockIdx.x;
  if (gridDim.x % 8 == 0) bx = (bx & 7) * (int)(gridDim.x / 8) + (bx >> 3);
  const int qtile = bx * 4 + wave, h = blockIdx.y, b = blockIdx.z;
  const int blk = qtile / p.tpb, qbase = (qtile - blk * p.tpb) * 64;
  if (blk >= nblocks) return;                 // no workgroup barriers below
  const int32_t *cnts = p.counts + (size_t)b * nblocks;
  const int32_t *lst = p.lists + (size_t)b * nblocks * p.cap;
  const int qcnt = __builtin_amdgcn_readfirstlane(min(cnts[blk] - qbase, 64));   // fill of the query tile
  if (qcnt <= 0) return;
  const int R = blk / p.nbw, C = blk % p.nbw;

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *vlds = smem + wave * 16384;  // two V tiles, row-major [key][64] bf16, swizzled
  const uint32_t lds_base = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)vlds);

  const char *qb = reinterpret_cast<const char *>(p.q + b * p.qsb + h * p.qsh);
  const char *kb = reinterpret_cast<const char *>(p.k + b * p.qsb + h * p.qsh);
  const char *vb = reinterpret_cast<const char *>(p.v + b * p.qsb + h * p.qsh);
  const uint32_t rowB = (uint32_t)p.qst * 2u;

  // token of slot `lane` of the run that starts at `base` in a block's list; slots beyond the
  // run's fill repeat its first slot (a valid row: its logits are masked, its weights are zero,
  // its output is not stored)
  // blk2 < 0: the global tokens after the first, tokens 1 .. n_global-1, as a list of their own
  auto slot_token = [&](int blk2, int base, int cnt) {
    const int slot = base + (lane < cnt ? lane : 0);
    return blk2 < 0 ? 1 + slot : lst[(size_t)blk2 * p.cap + slot];
  };

  // ---- Q as B operand: lane (query l32 + 32*nt, half hh) holds channels 32*hh + 8*s + j
  const int qtok = slot_token(blk, qbase, qcnt);
  bf16x8 qf[2][4];
  int qrow[2];
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    qrow[nt] = __shfl(qtok, l32 + 32 * nt);
    const char *row = qb + (size_t)qrow[nt] * rowB + 64 * hh;
#pragma unroll
    for (int s = 0; s < 4; s++) qf[nt][s] = *reinterpret_cast<const bf16x8 *>(row + 16 * s);
  }

  // transposed V reads (layout argument in ns_attn_mfma.hip)
  unsigned char *vrd[2][2];
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);
      const int off = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
      vrd[0][half] = vlds + off;
      vrd[1][half] = vlds + (off ^ 64);
    }
  }
  const uint32_t vchunk = 16u * ((lane & 7) ^ (((lane >> 4) & 1) << 2));   // swizzled source chunk

  // ---- state initialised by the global token (key 0): m = its logit, l = 1, O = v_0
  float m[2], l[2];
  f32x16 o[2][2];
  {
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
      m[nt] = half_swap_sum(acc) * p.c;
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
  }

  // ---- non-empty neighbour blocks as a bit mask over the 3x3 positions
  // fills of the nine neighbour positions (0 where the grid ends): lane nb loads its own, the wave
  // then keeps all nine as scalars, so that walking the tiles needs no further loads of them
  int fill_lane = 0;
  if (lane < 9) {
    const int R2 = R + lane / 3 - 1, C2 = C + lane % 3 - 1;
    if (R2 >= 0 && R2 < p.nbh && C2 >= 0 && C2 < p.nbw) fill_lane = cnts[R2 * p.nbw + C2];
  }
  int fill9[9];
#pragma unroll
  for (int i = 0; i < 9; i++) fill9[i] = __builtin_amdgcn_readlane(fill_lane, i);
  uint32_t nbmask = 0;
#pragma unroll
  for (int i = 0; i < 9; i++) nbmask |= fill9[i] > 0 ? 1u << i : 0u;   // the query block itself is non-empty: mask != 0

  // The key tiles in order: neighbour blocks by position, the runs of a block in list order.
  int kblk = 0, kfill = 0, kbase = 0;         // current block, its fill, start of the current run
  bool globals_pending = p.n_global > 1;      // they come first
  auto have_next = [&]() { return kbase + 64 < kfill || globals_pending || nbmask != 0; };
  auto advance = [&]() {                       // only when have_next()
    if (kbase + 64 < kfill) { kbase += 64; return; }
    if (globals_pending) {
      globals_pending = false;
      kblk = -1; kfill = p.n_global - 1; kbase = 0;
      return;
    }
    const int nb = __builtin_ctz(nbmask);
    nbmask &= nbmask - 1;
    kblk = (R + nb / 3 - 1) * p.nbw + (C + nb % 3 - 1);
    kfill = fill9[0];
#pragma unroll
    for (int i = 1; i < 9; i++) kfill = nb == i ? fill9[i] : kfill;
    kbase = 0;
  };
  // The tile after the one described last: its fill and, per lane, the token of its slot (the load
  // of the token travels together with the requests issued just before it and is consumed a
  // tile later).  False when the walk is over.
  auto next_desc = [&](int &cnt, int &tok) {
    if (!have_next()) return false;
    advance();
    cnt = min(kfill - kbase, 64);
    tok = slot_token(kblk, kbase, cnt);
    return true;
  };
  // requests of a key tile whose slot tokens are known: V into an LDS buffer (first: the transfers
  // are older than the fragment loads, so when the fragments are there, V is too), K fragments
  // into registers
  auto request = [&](bf16x8 (&kf)[2][4], int buf, int tok) {
    // (the lane numbers of the exchanges below are computed here, from an untraceable copy of the
    // lane number: kept in ten registers across the loop, two of them were spilled, and their
    // reload between the transfers waited for every transfer just issued)
    const int ln = opaque(lane);
#pragma unroll
    for (int it = 0; it < 8; it++) {
      const uint32_t vt = (uint32_t)__shfl(tok, it * 8 + (ln >> 3));
      dma16(vb, vt * rowB + vchunk, lds_base + buf * 8192 + it * 1024);
    }
#pragma unroll
    for (int mt = 0; mt < 2; mt++) {
      const uint32_t kt = (uint32_t)__shfl(tok, (ln & 31) + 32 * mt);
      const char *row = kb + (size_t)kt * rowB + 64 * hh;
#pragma unroll
      for (int s = 0; s < 4; s++) kf[mt][s] = *reinterpret_cast<const bf16x8 *>(row + 16 * s);
    }
  };
  auto stage_a = [&](const bf16x8 (&kf)[2][4], int mt, int nt) {
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[mt][ks], qf[nt][ks], s, 0, 0, 0);
    return s;
  };
  auto stage_c = [&](int mt, int nt, const bf16x8 (&pf)[2], int buf) {
#pragma unroll
    for (int sp = 0; sp < 2; sp++)
#pragma unroll
      for (int dt = 0; dt < 2; dt++) {
        const int off = buf * 8192 + (2 * mt + sp) * 2048;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][0] + off));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vrd[dt][1] + off));
        const bf16x4 a = __builtin_bit_cast(bf16x4, lo), b2 = __builtin_bit_cast(bf16x4, hi);
        const bf16x8 vf = {a[0], a[1], a[2], a[3], b2[0], b2[1], b2[2], b2[3]};
        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], o[dt][nt], 0, 0, 0);
      }
  };
  // the logits of a tile (its K fragments are there): [nt][mt], missing keys masked
  auto logits = [&](const bf16x8 (&kf)[2][4], int cnt, f32x16 (&sv)[2][2]) {
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      sv[nt][0] = stage_a(kf, 0, nt);
      sv[nt][1] = stage_a(kf, 1, nt);
      if (cnt < 64) {
        // register e of a 32x32 block is key 8*(e/4) + 4*hh + e%4 (+32 for the second block)
#pragma unroll
        for (int e = 0; e < 16; e++) {
          const int key = 8 * (e >> 2) + 4 * hh + (e & 3);
          sv[nt][0][e] = key < cnt ? sv[nt][0][e] : -INFINITY;
          sv[nt][1][e] = key + 32 < cnt ? sv[nt][1][e] : -INFINITY;
        }
      }
    }
  };
  // weights and output product of a tile from its logits; V is in LDS buffer buf
  auto weigh = [&](const f32x16 (&sv)[2][2], int buf) {
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const f32x16 &s0 = sv[nt][0], &s1 = sv[nt][1];
      float mx0 = fmaxf(s0[0], s0[1]), mx1 = fmaxf(s1[0], s1[1]);
#pragma unroll
      for (int e = 2; e < 16; e += 2) {
        mx0 = fmaxf(fmaxf(mx0, s0[e]), s0[e + 1]);
        mx1 = fmaxf(fmaxf(mx1, s1[e]), s1[e + 1]);
      }
      // the tile holds at least one key, and m starts finite: m_new is finite
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
        pa[e >> 3][e & 7] = ka[0]; pa[e >> 3][(e & 7) + 1] = ka[1];
        pb[e >> 3][e & 7] = kb2[0]; pb[e >> 3][(e & 7) + 1] = kb2[1];
      }
      l[nt] = __builtin_fmaf(l[nt], alpha, ls);
#pragma unroll
      for (int e = 0; e < 16; e++) { o[0][nt][e] *= alpha; o[1][nt][e] *= alpha; }
      stage_c(0, nt, pa, buf);
      stage_c(1, nt, pb, buf);
    }
  };

  // The walk.  A tile's logits come first: after them its K fragments are dead, and the next
  // tile's requests go out into the same registers (and the other V buffer) while the weights and
  // the output product of this one are computed.  Nothing with a register result is in flight
  // while a tile's fragments are waited for except the next token load, so no wait drains requests
  // that were just issued.
  bf16x8 kf[2][4];
  int cnt_cur = 0, tok_cur = 0, cnt_nxt = 0, tok_nxt = 0;
  next_desc(cnt_cur, tok_cur);                 // (the query block's own run is not empty: there is a first tile)
  request(kf, 0, tok_cur);
  bool has_nxt = next_desc(cnt_nxt, tok_nxt);
  int buf = 0;
  while (true) {
    f32x16 sv[2][2];
    logits(kf, cnt_cur, sv);
    // An ordering point that depends on the last logit tile, i.e. on the fragment load issued last:
    // every request of this tile is older than that load, so once it has returned the tile's V is
    // in LDS.  No LDS read below may be issued before this point, no transfer above it after it.
    {
      float t = sv[1][1][15];
      asm volatile("" : "+v"(t) :: "memory");
      sv[1][1][15] = t;
    }
    bool has_n2 = false;
    int cnt_n2 = 0, tok_n2 = 0;
    if (has_nxt) {
      request(kf, buf ^ 1, tok_nxt);
      has_n2 = next_desc(cnt_n2, tok_n2);
    }
    weigh(sv, buf);
    // the tile's LDS reads have returned before a transfer into its buffer is requested
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (!has_nxt) break;
    cnt_cur = cnt_nxt;
    cnt_nxt = cnt_n2; tok_nxt = tok_n2; has_nxt = has_n2;
    buf ^= 1;
  }

  // ---- normalise and store the rows that exist: lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3
  char *ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);
#pragma unroll
  for (int nt = 0; nt < 2; nt++) {
    const float inv = 1.f / half_swap_sum(l[nt]);
    if (l32 + 32 * nt >= qcnt) continue;
    char *row = ob + (size_t)qrow[nt] * (size_t)(p.ost * 2) + 8 * hh;
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

bool ragged_attn_supported(const ns_attn_desc &d) {
  return d.dtype == NS_BF16 && d.head_dim == 64 && d.radius == 1 && d.n_global >= 1 &&
         d.scale > 0.f && d.heads <= 65535 && d.batch <= 65535 &&
         (long long)d.tokens * d.q_stride_t * 2 < 0x7fffffffLL &&
         (long long)d.tokens * d.out_stride_t * 2 < 0x7fffffffLL;
}

ns_status launch_attn_ragged(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  RaggedParams p;
  p.q = static_cast<const uint16_t *>(a.q);
  p.k = static_cast<const uint16_t *>(a.k);
  p.v = static_cast<const uint16_t *>(a.v);
  p.out = static_cast<uint16_t *>(a.out);
  p.qsb = d.q_stride_b; p.qsh = d.q_stride_h; p.qst = d.q_stride_t;
  p.osb = d.out_stride_b; p.osh = d.out_stride_h; p.ost = d.out_stride_t;
  p.c = d.scale * kLog2e;
  p.nbh = a.geom.nbh; p.nbw = a.geom.nbw; p.cap = a.geom.cap;
  p.tpb = (p.cap + 63) / 64;
  p.n_global = d.n_global;
  p.heads = d.heads;
  p.lists = a.geom.lists; p.counts = a.geom.counts;
  if (!p.lists || !p.counts) return fail(NS_ERR_INVALID_ARG, "the list kernel was launched without block lists");
  const long long gx = ((long long)p.nbh * p.nbw * p.tpb + 3) / 4;
  if (gx > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "launch grid too large");
  hipLaunchKernelGGL(attn_mfma_ragged_kernel, dim3((unsigned)gx, d.heads, d.batch), dim3(256), 4 * 16384,
                     a.stream, p);
  return check_launch("attn_mfma_ragged_kernel");
}

}  // namespace ns
