// Persistent bf16 MFMA neighbourhood attention for patch queries on the full grid (gfx950).
// The default for full grids with at least two blocks per side where the sweep kernel does not apply
// (choose_patch_kernel in ns_api.hip); NSATTN_KERNEL=persist forces it.
//
// Same mathematics and register formulation as ns_attn_mfma.hip (transposed products, P kept in
// registers, fixed exponent reference with a checked fallback); what differs is how the chip is
// occupied.  One wave per SIMD (single-wave workgroups, 38 KB of LDS each) lives for the whole
// launch and walks a list of 64-query tiles.  Every global access of the steady state is an
// asynchronous global -> LDS transfer or a store, request-ordered:
//   K tile  in halves of 32 keys through a ring of three 4 KB half-slots (XOR swizzle), each half
//           read into registers right after the previous contents of those registers were last used,
//   V tile  in halves through a ring of two 8 KB slots, each half requested as soon as the half it
//           replaces has been read; ds_read_b64_tr_b16 at its use,
//   Q tile, k_0, v_0 of the NEXT query tile into a slot of their own, a whole query tile ahead.
// Requests do not stop at query-tile boundaries, so neither the per-query prologue nor any memory
// latency is exposed after the first tile of a wave.  No load with a register result is in
// flight while transfers are issued: the compiler's wait for such a load would also wait for
// every transfer issued after it (one in-order counter).
//
// Control flow.  The tile body contains no branches: a query tile is FIRST tile, a loop of MIDDLE
// tiles, LAST tile (three instantiations of one body), and everything that happens once per
// query tile (normalise, store, overflow check, next query's state) sits between them.  Ring
// positions are run-time scalars, so the body does not depend on how many key tiles a query tile
// has.  (Branches inside the body made the register allocator shuffle hundreds of values between
// the vector and accumulator files per tile in an earlier version.)
//
// Waits.  Vector memory operations complete in issue order, so "at most N outstanding"
// (s_waitcnt vmcnt(N)) means that everything but the N youngest has arrived.  Per key tile t the
// body issues, in this order: K(t+2) first half [4 requests], K(t+2) second half [4], V(t+1)
// second half [4], V(t+2) first half [4].  Before it reads the first half of K(t+1) and of V(t)
// it allows the 16 requests issued after those; likewise before the second halves.  The FIRST
// tile of a query tile additionally allows the 16 stores and 10 requests issued between the query
// tiles.  All of these are issued from asm, one instruction each, so the counts are exact.
#include "ns_common.h"
#include <type_traits>

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

constexpr int kStoresPerQuery = 16;   // 8-byte stores of one query tile's output
constexpr int kQueryRequests = 10;    // transfers of the next query tile: 8 (Q) + 1 (k_0) + 1 (v_0)
constexpr int kBodyWindow = 16;       // requests the body issues after the ones it is about to use
// LDS map of a wave, bytes
constexpr uint32_t KRING = 0;         // three half-slots of 4096
constexpr uint32_t VRING = 12288;     // two slots of 8192
constexpr uint32_t QSLOT = 28672;     // 64 query rows of 128 bytes, swizzled like K
constexpr uint32_t K0ROW = 36864;     // k_0 in the first 128 bytes of a 1 KB request
constexpr uint32_t V0ROW = 37888;     // v_0 likewise
constexpr uint32_t kLdsUsed = 38912;



#define NS_U(x) __builtin_amdgcn_readfirstlane(x)

template <int LOG2B>
__global__ __launch_bounds__(64, 2) void attn_mfma_persist_kernel(PersistParams p) {
  constexpr int B_ = 1 << LOG2B;
  constexpr int TPB = (B_ * B_) / 64;
  constexpr int TROWS = 64 / B_;
  const int lane = threadIdx.x;
  const int l32 = lane & 31, hh = lane >> 5;

  // ---- this wave's query tiles: XCD x owns a contiguous range of the (image-major) tile list,
  // its waves sweep that range together (tile = lo + slot + j*slots), so the XCD's L2 holds one
  // or two head-images' K and V at a time.  (Integer division runs on the vector ALU;
  // readfirstlane puts the uniform results back into scalar registers.)
  const int xcd = NS_U((int)blockIdx.x % p.xcds), slot = NS_U((int)blockIdx.x / p.xcds);
  const int slots = p.slots;
  const int lo = NS_U((int)((long long)p.tiles_total * xcd / p.xcds));
  const int hi = NS_U((int)((long long)p.tiles_total * (xcd + 1) / p.xcds));
  if (lo + slot >= hi) return;
  const int nq_wave = (hi - (lo + slot) + slots - 1) / slots;      // query tiles of this wave

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char *wlds = smem;
  const uint32_t lds_base = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)wlds);

  const uint32_t rowB = (uint32_t)p.qst * 2u;
  const uint32_t gridrowB = (uint32_t)p.grid_w * rowB;
  auto tile_off = [&](int i) { return (i >> LOG2B) * p.grid_w + (i & (B_ - 1)); };
  auto tile_base = [&](int R2, int C2, int sub) { return 1 + (R2 * B_ + sub * TROWS) * p.grid_w + C2 * B_; };

  // ---- per-lane constants
  // DMA source: LDS slot `lane` of request `it` holds row it*8 + lane/8, physical 16-byte chunk lane%8.
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
  const uint32_t krd0 = l32 * 128;
  uint32_t krd[4];
#pragma unroll
  for (int s = 0; s < 4; s++) krd[s] = krd0 + 16 * ((4 * hh + s) ^ ((l32 >> 1) & 7));
  // V transposed reads (see ns_attn_mfma.hip for the layout argument)
  uint32_t vrd[2][2];
  {
    const int g = lane >> 4, s = lane & 15;
    const int dbyte = (16 * (g & 1) + 4 * (s & 3)) * 2;
#pragma unroll
    for (int half = 0; half < 2; half++) {
      const int key = 8 * half + 4 * hh + (s >> 2);
      const int off = key * 128 + (dbyte ^ (((key >> 1) & 1) << 6));
      vrd[0][half] = VRING + off;
      vrd[1][half] = VRING + (off ^ 64);
    }
  }
  const uint32_t qoff0 = (uint32_t)tile_off(l32) * rowB + 64u * hh;   // K rows straight from global memory (redo path)

  // ---- query tiles and key tiles as scalar descriptors
  struct Query {
    int ntiles, R0, C0, ncols, R, C, qsub;
    const char *qb, *kb, *vb;
    char *ob;
  };
  auto open_query = [&](Query &c, int j) {          // j-th query tile of this wave, clamped to the last
    // (the slot is rotated from one query tile to the next, so that a wave does not stay in one
    // block column: border columns have fewer key tiles)
    const int jj = min(j, nq_wave - 1);
    const int base = lo + jj * slots;
    const int width = min(slots, hi - base);
    const int t = base + NS_U((slot + 37 * jj) % width);
    const int img = NS_U(t / p.tiles_per_image), rem = t - img * p.tiles_per_image;
    const int b = NS_U(img / p.heads), h = img - b * p.heads;
    const int blk = rem / TPB;               // TPB is a power of two
    c.qsub = rem % TPB;
    c.R = NS_U(blk / p.nbw); c.C = blk - c.R * p.nbw;
    c.R0 = max(c.R - 1, 0); c.C0 = max(c.C - 1, 0);
    const int R1 = min(c.R + 1, p.nbh - 1), C1 = min(c.C + 1, p.nbw - 1);
    c.ncols = C1 - c.C0 + 1;
    c.ntiles = (R1 - c.R0 + 1) * c.ncols * TPB;
    const int64_t ho = b * p.qsb + h * p.qsh;
    c.qb = reinterpret_cast<const char *>(p.q + ho);
    c.kb = reinterpret_cast<const char *>(p.k + ho);
    c.vb = reinterpret_cast<const char *>(p.v + ho);
    c.ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);
  };
  struct Tile { const char *kb, *vb; };     // K and V rows of key 0 of a key tile
  auto key_tile = [&](const Query &c, int i) {
    const int sub = i & (TPB - 1), nbi = i / TPB;
    const int dR = (nbi >= c.ncols) + (nbi >= 2 * c.ncols);
    const uint32_t off = (uint32_t)tile_base(c.R0 + dR, c.C0 + nbi - dR * c.ncols, sub) * rowB;
    Tile t;
    t.kb = c.kb + off; t.vb = c.vb + off;
    return t;
  };
  // half: 0 = keys 0..31 (requests 0..3), 1 = keys 32..63; dst: byte offset of the 4 KB destination
  auto dma_k_half = [&](const Tile &t, int half, uint32_t dst) {
#pragma unroll
    for (int i = 0; i < 4; i++)
      dma16(t.kb + dstep(4 * half + i), dma_koff[i & 1], lds_base + KRING + dst + i * 1024);
  };
  auto dma_v_half = [&](const Tile &t, int par, int half) {
#pragma unroll
    for (int it = 4 * half; it < 4 * half + 4; it++)
      dma16(t.vb + dstep(it), dma_voff, lds_base + VRING + par * 8192 + it * 1024);
  };
  // the query tile's rows (laid out and swizzled like a K tile) and the global token's key / value rows
  auto dma_query = [&](const Query &c) {            // kQueryRequests requests
    const char *t = c.qb + (uint32_t)tile_base(c.R, c.C, c.qsub) * rowB;
#pragma unroll
    for (int it = 0; it < 8; it++) dma16(t + dstep(it), dma_koff[it & 1], lds_base + QSLOT + it * 1024);
    dma16(c.kb, 16u * (lane & 7), lds_base + K0ROW);
    dma16(c.vb, 16u * (lane & 7), lds_base + V0ROW);
  };

  // ---- register state
  bf16x8 qf[2][4];                 // Q fragments of the current query tile
  bf16x8 kA[4], kB[4];             // K fragments: keys 0..31 / 32..63 of a key tile
  f32x16 o[2][2];
  float m[2], l[2], nm[2], la[2][2];

  // Q fragments out of the query slot: lane (query l32 + 32*nt, half hh), logical chunks 4*hh + s
  auto read_query = [&]() {
#pragma unroll
    for (int nt = 0; nt < 2; nt++)
#pragma unroll
      for (int s = 0; s < 4; s++) qf[nt][s] = *(lds_bf16x8_ptr)(wlds + QSLOT + nt * 4096 + krd[s]);
  };
  auto read_k_half = [&](bf16x8 (&kf)[4], uint32_t off) {     // off: byte offset of the half-slot
#pragma unroll
    for (int s = 0; s < 4; s++) kf[s] = *(lds_bf16x8_ptr)(wlds + KRING + krd[s] + off);
  };
  auto stage_a = [&](const bf16x8 (&kf)[4], int nt) {
    f32x16 s = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 4; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[nt][ks], s, 0, 0, 0);
    return s;
  };
  // The global token initialises the state: m = its logit (the fixed exponent reference), l = 1,
  // O = v_0.  k0: channels 32*hh + 8*s + j, i.e. the fragment of a key tile whose 32 rows are all
  // k_0, so every register of its product with Q is q . k_0: the reference comes out of the same
  // MFMA as all the other logits.  v0: channels 32*dt + 8*ig + 4*hh + e.
  auto init_state = [&](const bf16x8 (&k0)[4], const u32x2 (&v0)[2][4]) {
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
        const bf16x4 v4 = __builtin_bit_cast(bf16x4, v0[dt][ig]);
#pragma unroll
        for (int e = 0; e < 4; e++) {
          o[dt][0][4 * ig + e] = (float)v4[e];
          o[dt][1][4 * ig + e] = (float)v4[e];
        }
      }
  };
  auto init_state_lds = [&]() {
    bf16x8 k0[4];
    u32x2 v0[2][4];
#pragma unroll
    for (int s = 0; s < 4; s++) k0[s] = *(lds_bf16x8_ptr)(wlds + K0ROW + 64 * hh + 16 * s);
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int ig = 0; ig < 4; ig++)
        v0[dt][ig] = *(u32x2 __attribute__((address_space(3))) *)(wlds + V0ROW + 64 * dt + 16 * ig + 8 * hh);
    init_state(k0, v0);
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
  // O^T[:, nt] += V^T[:, keys 32*mt ..] P^T; voffs: V ring slot in bytes
  auto stage_c = [&](int mt, int nt, const bf16x8 (&pf)[2], uint32_t voffs) {
#pragma unroll
    for (int sp = 0; sp < 2; sp++)
#pragma unroll
      for (int dt = 0; dt < 2; dt++) {
        const uint32_t off = voffs + (2 * mt + sp) * 2048;
        const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(wlds + vrd[dt][0] + off));
        const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(wlds + vrd[dt][1] + off));
        const bf16x4 a = __builtin_bit_cast(bf16x4, lo4), b2 = __builtin_bit_cast(bf16x4, hi4);
        const bf16x8 vf = {a[0], a[1], a[2], a[3], b2[0], b2[1], b2[2], b2[3]};
        o[dt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sp], o[dt][nt], 0, 0, 0);
      }
  };

  // ---- the flattened (query tile, key tile) sequence.  cq: query tile being computed; nq: the
  // one after it; the producer position (pq, pi) is three key tiles ahead of the consumer and
  // therefore in cq or nq.  d1 / d2: key tiles t+1 and t+2 of the current key tile t.
  Query cq, nq, pq;
  int qj = 0;                        // index of cq among this wave's query tiles
  open_query(cq, 0);
  open_query(nq, 1);
  pq = cq;
  int pi = 0;
  auto next_tile = [&]() {           // descriptor at the producer position, then advance it (no branches)
    const Tile t = key_tile(pq, pi);
    pi++;
    const bool wrap = pi == pq.ntiles;
    pi = wrap ? 0 : pi;
    pq.ntiles = wrap ? nq.ntiles : pq.ntiles;
    pq.R0 = wrap ? nq.R0 : pq.R0;
    pq.C0 = wrap ? nq.C0 : pq.C0;
    pq.ncols = wrap ? nq.ncols : pq.ncols;
    pq.kb = wrap ? nq.kb : pq.kb;
    pq.vb = wrap ? nq.vb : pq.vb;
    return t;
  };
  Tile d0 = next_tile(), d1 = next_tile(), d2;
  int par = 0;                       // V ring slot of the current key tile t
  // K ring: with ka = 2t mod 3, half-slot ka holds K(t+1) second half, ka+2 its first half, and
  // ka+1 (mod 3) is free
  int ka = 0;
  auto mod3 = [](int x) { return x >= 3 ? x - 3 : x; };

  // Everything key tile t0 needs and everything the steady state would have requested before it
  // starts; all of it has landed on return.
  auto prime = [&](const Tile &t0, const Tile &t1) {
    const uint32_t hfree = mod3(ka + 1) * 4096u, hfirst = mod3(ka + 2) * 4096u, hsecond = ka * 4096u;
    dma_k_half(t0, 0, hfree);
    dma_k_half(t0, 1, hfirst);
    dma_v_half(t0, par, 0);
    dma_v_half(t0, par, 1);
    wait_vm<0>();
    read_k_half(kA, hfree);
    read_k_half(kB, hfirst);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    dma_k_half(t1, 0, hfirst);
    dma_k_half(t1, 1, hsecond);
    dma_v_half(t1, 1 - par, 0);
    wait_vm<0>();
  };

  f32x16 s00;
  bf16x8 p3[2];                      // weights of the previous key tile's last sub-block (its stage C is deferred)

  // One key tile.  FIRST / LAST: first / last key tile of a query tile.
  auto tile = [&](auto first_tag, auto last_tag) {
    constexpr bool FIRST = decltype(first_tag)::value, LAST = decltype(last_tag)::value;
    constexpr int W = kBodyWindow + (FIRST ? kStoresPerQuery + kQueryRequests : 0);
    const uint32_t hfree = mod3(ka + 1) * 4096u, hfirst = mod3(ka + 2) * 4096u, hsecond = ka * 4096u;
    const uint32_t vcur = par * 8192u, vnext = 8192u - vcur;
    d2 = next_tile();
    bf16x8 p0[2], p1[2], p2[2];
    // step 0
    dma_k_half(d2, 0, hfree);                        // K(t+2) keys 0..31
    const f32x16 s01 = stage_a(kA, 1);
    stage_b(s00, 0, p0);
    if (!FIRST) stage_c(1, 1, p3, vnext);            // previous tile's last sub-block (keys 32..63 of its V)
    // step 1: the first halves of K(t+1) and V(t) have landed
    wait_vm<W>();
    read_k_half(kA, hfirst);                         // K(t+1) keys 0..31
    dma_k_half(d2, 1, hfirst);                       // K(t+2) keys 32..63 take their place
    dma_v_half(d1, 1 - par, 1);                      // V(t+1) second half: that half was last read in step 0
    const f32x16 s10 = stage_a(kB, 0);
    stage_b(s01, 1, p1);
    stage_c(0, 0, p0, vcur);
    // step 2
    const f32x16 s11 = stage_a(kB, 1);
    stage_b(s10, 0, p2);
    stage_c(0, 1, p1, vcur);
    // step 3: the second halves of K(t+1) and V(t) have landed
    wait_vm<W>();
    read_k_half(kB, hsecond);                        // K(t+1) keys 32..63
    dma_v_half(d2, par, 0);                          // V(t+2) first half: that half was last read in step 2
    if (!LAST) s00 = stage_a(kA, 0);                 // first sub-block of the next key tile
    stage_b(s11, 1, p3);
    stage_c(1, 0, p2, vcur);
    if (LAST) stage_c(1, 1, p3, vcur);
    d0 = d1; d1 = d2;
    par ^= 1;
    ka = mod3(ka + 2);
  };
  using T = std::true_type;
  using F = std::false_type;

  // ---- prologue: the only place where this wave waits for a full round trip
  dma_query(cq);
  prime(d0, d1);
  read_query();
  init_state_lds();
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the slot has been read: the next query tile may land in it
  dma_query(nq);
  s00 = stage_a(kA, 0);

  while (true) {
    tile(T{}, F{});
    for (int i = cq.ntiles - 2; i > 0; i--) tile(F{}, F{});
    tile(F{}, T{});

    // ---- the query tile is complete
    l[0] += la[0][0] + la[0][1];
    l[1] += la[1][0] + la[1][1];
    float big = fmaxf(fabsf(l[0]), fabsf(l[1]));
#pragma unroll
    for (int i = 0; i < 16; i++)
      big = fmaxf(fmaxf(big, fmaxf(fabsf(o[0][0][i]), fabsf(o[0][1][i]))),
                  fmaxf(fabsf(o[1][0][i]), fabsf(o[1][1][i])));
    const bool bad = __any(!(big < 1e30f));
    const int qbase = tile_base(cq.R, cq.C, cq.qsub);
    auto store = [&]() {             // lane (query, hh) owns channels 32*dt + 8*ig + 4*hh + 0..3; kStoresPerQuery stores
#pragma unroll
      for (int nt = 0; nt < 2; nt++) {
        const float inv = 1.f / half_swap_sum(l[nt]);
        char *row = cq.ob + (size_t)(qbase + tile_off(l32 + 32 * nt)) * (size_t)(p.ost * 2) + 8 * hh;
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
          for (int ig = 0; ig < 4; ig++) {
            u32x2 u = {pack_bf16(o[dt][nt][4 * ig] * inv, o[dt][nt][4 * ig + 1] * inv),
                       pack_bf16(o[dt][nt][4 * ig + 2] * inv, o[dt][nt][4 * ig + 3] * inv)};
            store8(row + 64 * dt + 16 * ig, u);
          }
      }
    };
    store();
    if (bad) {
      // ---- a weight overflowed: redo this query tile with a running maximum, fragments straight
      // from global memory, V staged through ring slot 0; then restart the request pipeline at
      // the next key tile (d0) and store again.
      wait_vm<0>();
      {
        bf16x8 k0[4];
        u32x2 v0[2][4];
#pragma unroll
        for (int s = 0; s < 4; s++) k0[s] = *reinterpret_cast<const bf16x8 *>(cq.kb + 64 * hh + 16 * s);
#pragma unroll
        for (int dt = 0; dt < 2; dt++)
#pragma unroll
          for (int ig = 0; ig < 4; ig++)
            v0[dt][ig] = *reinterpret_cast<const u32x2 *>(cq.vb + 8 * hh + 64 * dt + 16 * ig);
        init_state(k0, v0);
      }
      for (int i = 0; i < cq.ntiles; i++) {
        const Tile t = key_tile(cq, i);
        bf16x8 kt[2][4];
        const uint32_t kstep = (32 >> LOG2B) * gridrowB;
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
#pragma unroll
          for (int s = 0; s < 4; s++)
            kt[mt][s] = *reinterpret_cast<const bf16x8 *>(t.kb + mt * kstep + qoff0 + 16 * s);
        dma_v_half(t, 0, 0);
        dma_v_half(t, 0, 1);
        wait_vm<0>();                 // also the K fragments above
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
          const f32x16 s0 = stage_a(kt[0], nt), s1 = stage_a(kt[1], nt);
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
          stage_c(0, nt, pa, 0);
          stage_c(1, nt, pb, 0);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // V reads done before the next transfer into the slot
      }
      store();
      // the query slot already holds the next query tile (requested before this query tile
      // began, drained above); restart the key-tile requests at the next key tile
      prime(d0, d1);
    }
    if (++qj >= nq_wave) break;

    // ---- next query tile: its Q, k_0, v_0 were requested a whole query tile ago (they are older
    // than everything the waits of this query tile's second key tile allowed to be in flight)
    cq = nq;
    open_query(nq, qj + 1);
    read_query();
    init_state_lds();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    dma_query(nq);                   // always issued (clamped to the last query tile): the FIRST tile counts on it
    s00 = stage_a(kA, 0);
  }
  wait_vm<0>();                      // requests past the end of the sequence (they repeat its last key tile)
}

}  // namespace

bool persist_attn_supported(const ns_attn_desc &d) {
  // every query tile needs at least 4 key tiles: its FIRST and LAST tile are different code, and
  // the request pipeline never runs more than one query tile ahead
  return mfma_attn_supported(d) && d.grid_h / d.block >= 2 && d.grid_w / d.block >= 2;
}

ns_status launch_attn_persist(const AttnArgs &a) {
  const ns_attn_desc &d = a.d;
  const int num_cus = device_cu_count();
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
  static_assert(kLdsUsed <= 40960, "LDS map");
  const size_t lds = 40960;                  // a quarter of a CU's LDS: four workgroups per CU, one per SIMD
  if (d.block == 8)
    hipLaunchKernelGGL(attn_mfma_persist_kernel<3>, dim3(p.num_wgs), dim3(64), lds, a.stream, p);
  else
    hipLaunchKernelGGL(attn_mfma_persist_kernel<4>, dim3(p.num_wgs), dim3(64), lds, a.stream, p);
  return check_launch("attn_mfma_persist_kernel");
}

}  // namespace ns
