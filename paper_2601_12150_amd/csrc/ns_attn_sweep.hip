// bf16 MFMA neighbourhood attention for 8x8 blocks (and 4x4, 2x2 blocks on 8x8 tiles): a workgroup
// sweeps a row of query blocks and shares every key tile among the query blocks that need it (gfx950).
//
// Why.  With one wave per query block and private key tiles, every K and V tile is fetched from
// L2 nine times (once per query block of its neighbourhood); measured, that L2 -> LDS traffic
// (about 1 GB per launch on a 128 x 128 grid with batch 2 and 16 heads) costs as much time as
// the arithmetic.  Here a workgroup of 4 waves owns one row of blocks of one (batch, head) image.
// It walks the key blocks of the three block rows R-1, R, R+1 column by column; each key tile is
// brought into LDS once (direct global -> LDS transfers, XOR-swizzled, 3-slot ring) and used by
// the query blocks of columns c-1, c, c+1.  Wave w owns query blocks w, w+4, w+8, ...: a block q
// is busy during columns q-1 .. q+1, the wave then has one column off, in which it normalises
// and stores q and loads the rows of q+4.  So three of the four waves compute at any time, every
// key tile costs a third of the L2 traffic, and with two workgroups per CU (two waves per SIMD)
// the off-time of one wave is the other's compute time.
//
// Mathematics and register formulation are those of ns_attn_mfma.hip: S^T = K Q^T and
// O^T += V^T P^T with v_mfma_f32_32x32x16_bf16, P kept in registers, the global token's logit as
// fixed exponent reference, a check for overflow at the end of each query block and a redo with
// a running maximum for the (rare) blocks that fail it.
//
// The global (CLS) query rides along: it attends to every key, and every key tile of block row R
// passes through the LDS of strip R exactly once.  In column c the wave that has its column off,
// (c+2) mod 4, multiplies that tile with q_0 as well (the same two MFMA products with q_0 in every
// column of the B operand), keeps a running (max, sum, weighted V sum) for the global query in
// LDS and writes the raw logits.  Each wave leaves one partial record per strip in the format of
// the chunked row kernel; cls_combine_kernel merges them.  K and V are thus read once per launch
// instead of twice.
//
// Synchronisation: one s_barrier per key tile.  Each wave issues a quarter of a tile's transfers
// and waits for its own share (vector memory operations complete in issue order, so
// "at most N outstanding" means all but the N youngest have arrived); the barrier then makes the
// tile visible to all and, at the same time, tells that everybody is done with the slot that
// the next transfer overwrites.
#include "ns_common.h"

namespace ns {

namespace {

struct SweepParams {
  const uint16_t *q, *k, *v;
  uint16_t *out;
  int64_t qsb, qsh, qst, osb, osh, ost;
  float c;              // scale * log2(e)
  int grid_h, grid_w, nbh, nbw;   // blocks per side: ceil(grid / 8)
  int heads;
  int strips;           // batch * heads * nbh
  int num_cus;
  int tokens;
  int n_global;         // G leading global tokens, 1 .. 8 (their K and V rows sit in LDS for the whole strip)
  float scale;
  float *cls_logits;    // [B,H,T] raw logits of the global query, or NULL
  float *cls_partials;  // [B,H,4*nbh,66] softmax partials of the global query, or NULL: no global row
};

typedef s16x4 __attribute__((address_space(3))) *lds_s16x4_ptr;
typedef bf16x8 __attribute__((address_space(3))) *lds_bf16x8_ptr;

constexpr uint32_t kSlot = 16384;     // one key tile: K [64][64] bf16, then V [64][64] bf16
constexpr uint32_t kVOff = 8192;
constexpr int kSlots = 3;
constexpr uint32_t kK0Row = 3 * 16384;         // k_0 in the first 128 bytes of a 1 KB transfer
constexpr uint32_t kV0Row = 3 * 16384 + 1024;  // v_0 likewise
constexpr uint32_t kQ0Row = 3 * 16384 + 2048;  // q_0 likewise
constexpr uint32_t kClsState = 3 * 16384 + 3072;   // per wave 512 B: o[64], m, l of the global query's partial
constexpr uint32_t kClsLogit = 3 * 16384 + 3072 + 4 * 512;   // per wave 256 B: a tile's 64 logits
constexpr float kEmptyMax = -1e30f;
constexpr float kMasked = -1e30f;     // logit of a key that does not exist (edge blocks of a grid 8 does not divide)


#define NS_U(x) __builtin_amdgcn_readfirstlane(x)

// grid: one workgroup of 256 threads per strip (row of 8x8 tiles of one image).  EDGE: the grid
// has short tiles at its right or bottom edge (a side that 8 does not divide).  W: side of the
// token blocks that define the neighbourhood, a divisor of 8.  For W < 8 the 8x8 tiles stay the
// unit of work (a query tile still meets the 3x3 tiles around it, which contain the 3x3 blocks
// around each of its tokens), and every logit of a (query, key) pair whose blocks are not
// neighbours is masked.
template <bool EDGE, int W>
__global__ __launch_bounds__(256, 2) void attn_sweep_kernel(SweepParams p) {
  const int tid = threadIdx.x, wave = NS_U(tid >> 6), lane = tid & 63;
  const int l32 = lane & 31, hh = lane >> 5;

  // consecutive strips (neighbouring block rows of one image share two of their three key rows)
  // go to the same XCD: workgroups are dealt round-robin to the 8 XCDs
  int sid = blockIdx.x;
  if (p.strips % 8 == 0) sid = (sid & 7) * (p.strips / 8) + (sid >> 3);
  const int img = NS_U(sid / p.nbh), R = sid - img * p.nbh;
  const int b = NS_U(img / p.heads), h = img - b * p.heads;
  const char *qb = reinterpret_cast<const char *>(p.q + b * p.qsb + h * p.qsh);
  const char *kb = reinterpret_cast<const char *>(p.k + b * p.qsb + h * p.qsh);
  const char *vb = reinterpret_cast<const char *>(p.v + b * p.qsb + h * p.qsh);
  char *ob = reinterpret_cast<char *>(p.out + b * p.osb + h * p.osh);

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const uint32_t lds_base = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);

  const uint32_t rowB = (uint32_t)p.qst * 2u;
  const uint32_t gridrowB = (uint32_t)p.grid_w * rowB;
  // token (grid row 8*Rb + i/8, grid column 8*Cb + i%8) is row i of the tile of block (Rb, Cb)
  auto block_token = [&](int Rb, int Cb) { return p.n_global + Rb * 8 * p.grid_w + Cb * 8; };
  auto block_base = [&](int Rb, int Cb) { return (uint32_t)block_token(Rb, Cb) * rowB; };
  // Blocks at the right and bottom edge of a grid that 8 does not divide are short.  Their tiles
  // are filled up with copies of existing rows (the row and column index within the block are
  // clamped): a copied QUERY computes what its original computes and is stored to the same place
  // (same bits), a copied KEY gets the logit kMasked, i.e. the weight 0.
  const int hv_last = EDGE ? p.grid_h - 8 * (p.nbh - 1) : 8, wv_last = EDGE ? p.grid_w - 8 * (p.nbw - 1) : 8;   // 1 .. 8
  const int hvq = EDGE && R == p.nbh - 1 ? hv_last : 8;       // rows of this strip's query blocks
  auto tile_off = [&](int i, int hv, int wv) {
    return (uint32_t)(min(i >> 3, hv - 1) * p.grid_w + min(i & 7, wv - 1)) * rowB;
  };
  // logits of keys that do not exist: accumulator register e (key half mt) is key row 4*mt + e/4
  // and column 4*hh + e%4 of a block with hv rows and wv columns
  auto mask_keys = [&](f32x16 &sv, int mt, int hv, int wv) {
#pragma unroll
    for (int e = 0; e < 16; e++) sv[e] = (4 * mt + (e >> 2) >= hv || 4 * hh + (e & 3) >= wv) ? kMasked : sv[e];
  };
  // W < 8: logits of pairs whose WxW blocks are not neighbours.  The key tile lies (dr, dc) tiles
  // from the query tile; lane = query (tile row l32/8 + 4*nt, column l32%8), register e = key (tile
  // row 4*mt + e/4, column 4*hh + e%4); block indices relative to the query tile's first block.
  // (a copied query of a short tile sits where its original sits: wvq = columns of the query tile)
  auto mask_window = [&](f32x16 &sv, int mt, int nt, int dr, int dc, int wvq) {
    constexpr int n = 8 / W;
    const int rq = EDGE ? min((l32 >> 3) + 4 * nt, hvq - 1) : (l32 >> 3) + 4 * nt;
    const int cq = EDGE ? min(l32 & 7, wvq - 1) : (l32 & 7);
    const int ra = rq / W - n * dr + 1, ca = cq / W - n * dc + 1;
#pragma unroll
    for (int e = 0; e < 16; e++) {
      const bool ok = (unsigned)(ra - (4 * mt + (e >> 2)) / W) <= 2u && (unsigned)(ca - (4 * hh + (e & 3)) / W) <= 2u;
      sv[e] = ok ? sv[e] : kMasked;
    }
  };

  // ---- per-lane constants
  // transfers: request `it` of a tile is its rows 8*it .. 8*it+7 (one grid row of the block);
  // LDS slot `lane` holds row it*8 + lane/8, physical 16-byte chunk lane%8, which is logical chunk
  // (lane%8) ^ ((row>>1)&7) for K and (lane%8) ^ 4*((row>>1)&1) for V.  This wave issues requests
  // 2*wave and 2*wave+1 of K and of V; (row>>1)&7 = (4*(it&1) + (lane/8 >> 1)) & 7.
  const int drow = lane >> 3;
  const uint32_t dma_koff[2] = {drow * rowB + 16u * ((lane & 7) ^ ((drow >> 1) & 7)),
                                drow * rowB + 16u * ((lane & 7) ^ ((4 + (drow >> 1)) & 7))};
  const uint32_t dma_voff = drow * rowB + 16u * ((lane & 7) ^ (((drow >> 1) & 1) << 2));
  // K fragment reads: lane (row l32 [+32], half hh) needs logical chunks 4*hh + s
  uint32_t krd[4];
#pragma unroll
  for (int s = 0; s < 4; s++) krd[s] = l32 * 128 + 16 * ((4 * hh + s) ^ ((l32 >> 1) & 7));
  // V transposed reads (see ns_attn_mfma.hip for the layout argument)
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
  const uint32_t qoff0 = tile_off(l32, hvq, 8) + 64u * hh;
  const uint32_t qoff1 = tile_off(l32 + 32, hvq, 8) + 64u * hh;

  // ---- the key tiles of this strip, column by column
  const int r0 = max(R - 1, 0), r1 = min(R + 1, p.nbh - 1);
  const int nr = r1 - r0 + 1, ncols = p.nbw, steps = ncols * nr;
  // this wave's share (4 requests) of the transfers of the next key tile in column-major order
  // into the next ring slot; past the last tile it repeats that one (into a slot nobody reads)
  int ic = 0, ir = 0, islot = 0;     // column, row within the column and ring slot of the tile to request
  auto issue_next = [&]() {
    const uint32_t base = block_base(r0 + ir, ic);
    const uint32_t dst = lds_base + (uint32_t)islot * kSlot + (uint32_t)wave * 2048u;
    const int hvk = EDGE && r0 + ir == p.nbh - 1 ? hv_last : 8;
    // a short block's missing columns: the lanes of those columns fetch its last column instead
    uint32_t back = 0;
    if (EDGE && ic == ncols - 1 && wv_last < 8) back = (uint32_t)max(drow - (wv_last - 1), 0) * rowB;
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const char *src = kb + base + (size_t)min(2 * wave + j, hvk - 1) * gridrowB;
      dma16(src, dma_koff[j] - back, dst + j * 1024);
    }
#pragma unroll
    for (int j = 0; j < 2; j++) {
      const char *src = vb + base + (size_t)min(2 * wave + j, hvk - 1) * gridrowB;
      dma16(src, dma_voff - back, dst + kVOff + j * 1024);
    }
    islot = islot == kSlots - 1 ? 0 : islot + 1;
    const bool last = ic == ncols - 1 && ir == nr - 1;
    const bool wrap = ir == nr - 1;
    ic = last ? ic : (wrap ? ic + 1 : ic);
    ir = last ? ir : (wrap ? 0 : ir + 1);
  };

  // ---- register state of the query block in progress
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
  // Q fragments of query block qc by ordinary loads
  auto load_block = [&](int qc) {
    const char *t = qb + block_base(R, qc);
    uint32_t back = 0;                 // (l32 and l32 + 32 are in the same column of the block)
    if (EDGE && qc == ncols - 1 && wv_last < 8) back = (uint32_t)max((l32 & 7) - (wv_last - 1), 0) * rowB;
#pragma unroll
    for (int s = 0; s < 4; s++) {
      qf[0][s] = *reinterpret_cast<const bf16x8 *>(t + (qoff0 - back) + 16 * s);
      qf[1][s] = *reinterpret_cast<const bf16x8 *>(t + (qoff1 - back) + 16 * s);
    }
  };
  // The state the global token gives a query block: m = its logit (the fixed exponent reference),
  // l = 1, O = v_0.  k_0 and v_0 sit in LDS for the whole strip.  The k_0 fragment is that of a
  // key tile whose rows are all k_0, so every register of its product with Q is q . k_0.
  // Further global tokens (rows 1 .. G-1 of the same LDS areas) are added one by one with a
  // running maximum, so the reference becomes the largest of the global tokens' logits.
  auto init_block = [&]() {
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
  uint32_t badmask = 0;              // bit j: this wave's j-th query block has to be redone
  // Normalised rows of the finished block, packed: lane (query, hh) owns channels
  // 32*dt + 8*ig + 4*hh + 0..3.  Also notes whether a weight overflowed the fixed reference
  // (then some sum or output is not finite).
  u32x2 packed[2][2][4];
  auto finish_math = [&](int qc) {
    l[0] += la[0][0] + la[0][1];
    l[1] += la[1][0] + la[1][1];
    float big = fmaxf(fabsf(l[0]), fabsf(l[1]));
#pragma unroll
    for (int i = 0; i < 16; i++)
      big = fmaxf(fmaxf(big, fmaxf(fabsf(o[0][0][i]), fabsf(o[0][1][i]))),
                  fmaxf(fabsf(o[1][0][i]), fabsf(o[1][1][i])));
    if (__any(!(big < 1e30f))) badmask |= 1u << (qc >> 2);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const float inv = 1.f / half_swap_sum(l[nt]);
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int ig = 0; ig < 4; ig++)
          packed[nt][dt][ig] = u32x2{pack_bf16(o[dt][nt][4 * ig] * inv, o[dt][nt][4 * ig + 1] * inv),
                                     pack_bf16(o[dt][nt][4 * ig + 2] * inv, o[dt][nt][4 * ig + 3] * inv)};
    }
  };
  constexpr int kStores = 16;        // requests of store_block
  auto store_block = [&](int qc) {
    char *t = ob + (size_t)block_token(R, qc) * (size_t)(p.ost * 2);
#pragma unroll
    for (int nt = 0; nt < 2; nt++) {
      const int i = l32 + 32 * nt;
      const int wvq = EDGE && qc == ncols - 1 ? wv_last : 8;
      char *row = t + (size_t)(min(i >> 3, hvq - 1) * p.grid_w + min(i & 7, wvq - 1)) * (size_t)(p.ost * 2) + 8 * hh;
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int ig = 0; ig < 4; ig++) store8(row + 64 * dt + 16 * ig, packed[nt][dt][ig]);
    }
  };

  // ---- the global query's share of a key tile (see the head of the file).  State in LDS per
  // wave: o[64] in channel order, then the running maximum (log2 domain) and the sum.
  float *const cls_state = reinterpret_cast<float *>(smem + kClsState + wave * 512);
  float *const cls_logit = reinterpret_cast<float *>(smem + kClsLogit + wave * 256);
  float *const logit_row = p.cls_logits ? p.cls_logits + ((size_t)b * p.heads + h) * p.tokens : nullptr;
  auto cls_duty = [&](uint32_t slot, int col, bool with_global_key) {
    const int wvc = EDGE && col == ncols - 1 ? wv_last : 8;    // the tile is block (R, col): hvq rows, wvc columns
    // q_0 as B operand, the same in all 32 columns: channels 32*hh + 8*s + j
    bf16x8 q0f[4], kA[4], kB[4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
      q0f[t] = *(lds_bf16x8_ptr)(smem + kQ0Row + 64 * hh + 16 * t);
      kA[t] = *(lds_bf16x8_ptr)(smem + slot + krd[t]);
      kB[t] = *(lds_bf16x8_ptr)(smem + slot + 4096 + krd[t]);
    }
    f32x16 sa = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}, sb = sa;
#pragma unroll
    for (int ks = 0; ks < 4; ks++) {
      sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kA[ks], q0f[ks], sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kB[ks], q0f[ks], sb, 0, 0, 0);
    }
    if (EDGE && (hvq < 8 || wvc < 8)) {
      mask_keys(sa, 0, hvq, wvc);
      mask_keys(sb, 1, hvq, wvc);
    }
    // register e of sa is key 8*(e/4) + 4*hh + e%4 of the tile (sb: + 32), whatever the column
    if (logit_row) {
      if (l32 == 0) {
#pragma unroll
        for (int g = 0; g < 4; g++) {
          const f32x4 va = {sa[4 * g] * p.scale, sa[4 * g + 1] * p.scale, sa[4 * g + 2] * p.scale, sa[4 * g + 3] * p.scale};
          const f32x4 vb2 = {sb[4 * g] * p.scale, sb[4 * g + 1] * p.scale, sb[4 * g + 2] * p.scale, sb[4 * g + 3] * p.scale};
          *reinterpret_cast<f32x4 *>(cls_logit + 8 * g + 4 * hh) = va;
          *reinterpret_cast<f32x4 *>(cls_logit + 32 + 8 * g + 4 * hh) = vb2;
        }
      }
      // lane = key of the tile: token (grid row 8R + lane/8, grid column 8*col + lane%8); the lane of
      // a key that does not exist repeats the store of the key it copies
      // (addresses computed here, from an untraceable copy of the lane number: hoisted out of the
      // key-tile loop they cost three registers that the compute branch does not have, and their
      // reload from scratch memory waits for every transfer in flight)
      const int ln = opaque(lane);
      const int kr = min(ln >> 3, hvq - 1), kc = min(ln & 7, wvc - 1);
      const float x = cls_logit[8 * kr + kc];
      store4(logit_row + block_token(R, col) + kr * p.grid_w + kc, x);
    }
    float mx = fmaxf(sa[0], sb[0]);
#pragma unroll
    for (int e = 1; e < 16; e++) mx = fmaxf(mx, fmaxf(sa[e], sb[e]));
    mx = half_swap_max(mx) * p.c;
    float m2 = cls_state[64], l0 = cls_state[65];
    float k0logit = 0.f;
    if (with_global_key) {
      // key 0 (the global token itself) belongs to the first tile of the image
      bf16x8 k0[4];
#pragma unroll
      for (int t = 0; t < 4; t++) k0[t] = *(lds_bf16x8_ptr)(smem + kK0Row + 64 * hh + 16 * t);
      f32x16 s0 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 4; ks++) s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[ks], q0f[ks], s0, 0, 0, 0);
      k0logit = s0[0];
      mx = fmaxf(mx, k0logit * p.c);
      if (logit_row && lane == 0) store4(logit_row, k0logit * p.scale);
    }
    const float m_new = fmaxf(m2, mx);
    const float alpha = __builtin_amdgcn_exp2f(m2 - m_new), nmm = -m_new;
    float ls = 0.f;
    bf16x8 pa[2], pb[2];
#pragma unroll
    for (int e = 0; e < 16; e += 2) {
      const float a0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[e], p.c, nmm));
      const float a1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[e + 1], p.c, nmm));
      const float b0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sb[e], p.c, nmm));
      const float b1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sb[e + 1], p.c, nmm));
      ls += (a0 + a1) + (b0 + b1);
      const bf16x2 ka = __builtin_bit_cast(bf16x2, pack_bf16(a0, a1));
      const bf16x2 kb2 = __builtin_bit_cast(bf16x2, pack_bf16(b0, b1));
      pa[e >> 3][e & 7] = ka[0]; pa[e >> 3][(e & 7) + 1] = ka[1];
      pb[e >> 3][e & 7] = kb2[0]; pb[e >> 3][(e & 7) + 1] = kb2[1];
    }
    ls = half_swap_sum(ls);                       // the two half-waves hold different keys
    // O (one column's worth, the same in every column): channel 32*dt + 8*(e/4) + 4*hh + e%4
    f32x16 oc[2];
#pragma unroll
    for (int dt = 0; dt < 2; dt++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const f32x4 v = *reinterpret_cast<const f32x4 *>(cls_state + 32 * dt + 8 * g + 4 * hh);
#pragma unroll
        for (int e = 0; e < 4; e++) oc[dt][4 * g + e] = v[e] * alpha;
      }
    float pk0 = 0.f;
    if (with_global_key) {
      pk0 = __builtin_amdgcn_exp2f(__builtin_fmaf(k0logit, p.c, nmm));
      ls += pk0;
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          const u32x2 v2 = *(u32x2 __attribute__((address_space(3))) *)(smem + kV0Row + 64 * dt + 16 * g + 8 * hh);
          const bf16x4 v4 = __builtin_bit_cast(bf16x4, v2);
#pragma unroll
          for (int e = 0; e < 4; e++) oc[dt][4 * g + e] = __builtin_fmaf(pk0, (float)v4[e], oc[dt][4 * g + e]);
        }
    }
#pragma unroll
    for (int mt = 0; mt < 2; mt++)
#pragma unroll
      for (int sp = 0; sp < 2; sp++)
#pragma unroll
        for (int dt = 0; dt < 2; dt++) {
          const uint32_t off = slot + (2 * mt + sp) * 2048;
          const s16x4 lo4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smem + vrd[dt][0] + off));
          const s16x4 hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(smem + vrd[dt][1] + off));
          const bf16x4 a = __builtin_bit_cast(bf16x4, lo4), b2 = __builtin_bit_cast(bf16x4, hi4);
          const bf16x8 vf = {a[0], a[1], a[2], a[3], b2[0], b2[1], b2[2], b2[3]};
          oc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, mt == 0 ? pa[sp] : pb[sp], oc[dt], 0, 0, 0);
        }
    if (l32 == 0) {
#pragma unroll
      for (int dt = 0; dt < 2; dt++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          const f32x4 v = {oc[dt][4 * g], oc[dt][4 * g + 1], oc[dt][4 * g + 2], oc[dt][4 * g + 3]};
          *reinterpret_cast<f32x4 *>(cls_state + 32 * dt + 8 * g + 4 * hh) = v;
        }
      if (hh == 0) {
        cls_state[64] = m_new;
        cls_state[65] = __builtin_fmaf(l0, alpha, ls);
      }
    }
  };

  // ---- prologue: the first three key tiles are requested, the first has landed
  int qc = wave;                     // this wave's query block in progress
  if (wave == 0) {
    // the global tokens' rows, 8 lanes x 16 bytes each: LDS row r = token min(r, G-1)
    const uint32_t goff = (uint32_t)min(lane >> 3, p.n_global - 1) * rowB + 16u * (lane & 7);
    dma16(kb, goff, lds_base + kK0Row);
    dma16(vb, goff, lds_base + kV0Row);
    dma16(qb, 16u * (lane & 7), lds_base + kQ0Row);
  }
  cls_state[lane] = 0.f;             // this wave's partial of the global query: nothing seen yet
  if (lane < 2) cls_state[64 + lane] = lane == 0 ? kEmptyMax : 0.f;
  issue_next();
  issue_next();
  issue_next();
  wait_vm<8>();                     // k_0, v_0, q_0 and tile 0
  __syncthreads();
  // (loading and consuming the rows under ONE condition matters: the compiler places its waits
  // per program point, not per path, and a load that looks pending at the loop head would put a
  // full wait into every key tile)
  if (qc < ncols) {
    load_block(qc);
    init_block();
  }

  int c = 0, ri = 0, cslot = 0;      // column, row within the column and ring slot of key tile s
  // Two workgroups share a CU, and among waves of equal priority a SIMD issues the older one
  // first: the workgroup that arrived first runs at nearly full speed (measured 1.5 us per key
  // tile against 2.1 us for the other) and leaves the CU half empty once it is done.  The later
  // one (launch order: workgroups i and i + number of CUs share a CU) therefore raises its
  // priority for the rest of its strip once it is 3/8 through, so that both finish at about the
  // same time (measured: 6 % off the launch).
  const bool later = NS_U((int)(blockIdx.x / p.num_cus) & 1) != 0;
  const int boost_at = (steps * 3) >> 3;
  for (int s = 0; s < steps; s++) {
    if (later && s == boost_at) __builtin_amdgcn_s_setprio(3);
    const uint32_t slot = (uint32_t)cslot * kSlot;
    int extra = 0;                   // stores issued in this step
    if (qc < ncols && c + 1 >= qc && c <= qc + 1) {
      // ---- key tile s against this wave's query block
      bf16x8 kA[4], kB[4], p0[2], p1[2], p2[2], p3[2];
#pragma unroll
      for (int t = 0; t < 4; t++) {
        kA[t] = *(lds_bf16x8_ptr)(smem + slot + krd[t]);
        kB[t] = *(lds_bf16x8_ptr)(smem + slot + 4096 + krd[t]);
      }
      // (a short key block: its missing keys get the logit kMasked)
      const int hvk = EDGE && r0 + ri == p.nbh - 1 ? hv_last : 8, wvk = EDGE && c == ncols - 1 ? wv_last : 8;
      const bool edge = EDGE && (hvk < 8 || wvk < 8);
      const int dr = r0 + ri - R, dc = c - qc;
      const int wvq = EDGE && qc == ncols - 1 ? wv_last : 8;
      f32x16 s00 = stage_a(kA, 0);
      if (edge) mask_keys(s00, 0, hvk, wvk);
      if (W < 8) mask_window(s00, 0, 0, dr, dc, wvq);
      f32x16 s01 = stage_a(kA, 1);
      if (edge) mask_keys(s01, 0, hvk, wvk);
      if (W < 8) mask_window(s01, 0, 1, dr, dc, wvq);
      stage_b(s00, 0, p0);
      f32x16 s10 = stage_a(kB, 0);
      if (edge) mask_keys(s10, 1, hvk, wvk);
      if (W < 8) mask_window(s10, 1, 0, dr, dc, wvq);
      stage_b(s01, 1, p1);
      stage_c(0, 0, p0, slot);
      f32x16 s11 = stage_a(kB, 1);
      if (edge) mask_keys(s11, 1, hvk, wvk);
      if (W < 8) mask_window(s11, 1, 1, dr, dc, wvq);
      stage_b(s10, 0, p2);
      stage_c(0, 1, p1, slot);
      stage_b(s11, 1, p3);
      stage_c(1, 0, p2, slot);
      stage_c(1, 1, p3, slot);
      extra = 0;
    } else if (qc < ncols && c > qc + 1) {
      // ---- the column off: finish the block, start this wave's next one.  Order: request the
      // next block's rows, normalise the finished one, consume the rows (that wait also covers
      // every transfer issued so far), and only then store, so that no wait sees the stores
      // except the one below, which allows for them.
      const int qdone = qc;
      qc += 4;
      const bool next = qc < ncols;
      if (next) {
        load_block(qc);
        finish_math(qdone);
        init_block();
      } else {
        finish_math(qdone);
      }
      store_block(qdone);
      extra = kStores;
    }
    // the global query's share of the tile of this strip's own block row: the wave that has column c off
    if (p.cls_partials && ri == R - r0 && wave == ((c + 2) & 3)) {
      const bool first = R == 0 && c == 0;
      cls_duty(slot, c, first);
      if (logit_row) extra += first ? 2 : 1;
    }
    // tile s+1: this wave's share has landed (its share of tile s+2 and the stores above may still be in flight)
    switch (extra) {
      case 0: wait_vm<4>(); break;
      case 1: wait_vm<5>(); break;
      case 2: wait_vm<6>(); break;
      case kStores: wait_vm<4 + kStores>(); break;
      case kStores + 1: wait_vm<5 + kStores>(); break;
      default: wait_vm<6 + kStores>(); break;
    }
    // everybody's share of tile s+1 has landed; and everybody is done with tile s, whose slot tile s+3 takes
    __syncthreads();
    issue_next();
    cslot = cslot == kSlots - 1 ? 0 : cslot + 1;
    ri++;
    if (ri == nr) { ri = 0; c++; }
  }
  wait_vm<0>();
  if (p.cls_partials) {
    // this wave's partial of the global query's row: (max, sum, weighted V sum), natural-log units
    float *rec = p.cls_partials + ((((size_t)b * p.heads + h) * (4 * p.nbh)) + (size_t)R * 4 + wave) * kClsPartialFloats;
    rec[2 + lane] = cls_state[lane];
    if (lane == 0) {
      rec[0] = cls_state[64] * kLn2;
      rec[1] = cls_state[65];
    }
  }
  if (qc < ncols) {                  // the block whose last column was the strip's last
    finish_math(qc);
    store_block(qc);
  }
  __syncthreads();                   // the ring is free: each wave takes 16 KB of it below

  // ---- query blocks in which a weight overflowed (their stored rows are not finite): once more
  // with a running maximum, fragments straight from global memory, V staged through LDS
  const uint32_t mine = (uint32_t)wave * 16384u;
  for (int j = 0; badmask; j++, badmask >>= 1) {
    if (!(badmask & 1)) continue;
    const int qr = wave + 4 * j;
    load_block(qr);
    init_block();
    for (int cc = max(qr - 1, 0); cc <= min(qr + 1, ncols - 1); cc++)
      for (int rr = r0; rr <= r1; rr++) {
        const uint32_t base = block_base(rr, cc);
        const int hvk = EDGE && rr == p.nbh - 1 ? hv_last : 8, wvk = EDGE && cc == ncols - 1 ? wv_last : 8;
        bf16x8 kt[2][4];
#pragma unroll
        for (int mt = 0; mt < 2; mt++)
#pragma unroll
          for (int t = 0; t < 4; t++)
            kt[mt][t] = *reinterpret_cast<const bf16x8 *>(kb + base + tile_off(l32 + 32 * mt, hvk, wvk) + 64 * hh + 16 * t);
        const uint32_t back = (uint32_t)max(drow - (wvk - 1), 0) * rowB;
#pragma unroll
        for (int it = 0; it < 8; it++)
          dma16(vb + base + (size_t)min(it, hvk - 1) * gridrowB, dma_voff - back, lds_base + mine + kVOff + it * 1024);
        wait_vm<0>();               // also the K fragments above
#pragma unroll
        for (int nt = 0; nt < 2; nt++) {
          f32x16 s0 = stage_a(kt[0], nt), s1 = stage_a(kt[1], nt);
          if (EDGE && (hvk < 8 || wvk < 8)) {
            mask_keys(s0, 0, hvk, wvk);
            mask_keys(s1, 1, hvk, wvk);
          }
          if (W < 8) {
            const int wvq = EDGE && qr == ncols - 1 ? wv_last : 8;
            mask_window(s0, 0, nt, rr - R, cc - qr, wvq);
            mask_window(s1, 1, nt, rr - R, cc - qr, wvq);
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
    const uint32_t keep = badmask;
    finish_math(qr);                 // (its overflow note is void here)
    badmask = keep;
    store_block(qr);
  }
}

}  // namespace

bool sweep_attn_supported(const ns_attn_desc &d) {
  return d.dtype == NS_BF16 && d.head_dim == 64 && d.radius == 1 && d.n_global >= 1 && d.n_global <= 8 &&
         d.coords == nullptr &&
         (d.block == 8 || d.block == 4 || d.block == 2) && (d.grid_w + 7) / 8 <= 128 && d.scale > 0.f &&
         // tokens are addressed with 32-bit byte offsets from the (batch, head) base
         (long long)d.tokens * d.q_stride_t * 2 < 0x7fffffffLL &&
         (long long)d.tokens * d.out_stride_t * 2 < 0x7fffffffLL;
}

ns_status launch_attn_sweep(const AttnArgs &a, float *cls_logits, float *cls_partials) {
  const ns_attn_desc &d = a.d;
  SweepParams p;
  p.q = static_cast<const uint16_t *>(a.q);
  p.k = static_cast<const uint16_t *>(a.k);
  p.v = static_cast<const uint16_t *>(a.v);
  p.out = static_cast<uint16_t *>(a.out);
  p.qsb = d.q_stride_b; p.qsh = d.q_stride_h; p.qst = d.q_stride_t;
  p.osb = d.out_stride_b; p.osh = d.out_stride_h; p.ost = d.out_stride_t;
  p.c = d.scale * kLog2e;
  p.grid_h = d.grid_h;
  p.grid_w = d.grid_w;
  p.nbh = (d.grid_h + 7) / 8;
  p.nbw = (d.grid_w + 7) / 8;
  p.heads = d.heads;
  p.tokens = d.tokens;
  p.n_global = d.n_global;
  p.scale = d.scale;
  // the global query's row on the way: with one global token only (several take the row kernel)
  p.cls_logits = d.n_global == 1 ? cls_logits : nullptr;
  p.cls_partials = d.n_global == 1 ? cls_partials : nullptr;
  const long long strips = (long long)d.batch * d.heads * p.nbh;
  if (strips > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "launch grid too large");
  // a wave records the query blocks it has to redo in a 32-bit mask
  if (p.nbw > 128) return fail(NS_ERR_UNSUPPORTED, "more than 128 blocks per grid row");
  p.strips = (int)strips;
  p.num_cus = device_cu_count();
  typedef void (*kern_t)(SweepParams);
  static const kern_t kerns[3][2] = {{attn_sweep_kernel<false, 8>, attn_sweep_kernel<true, 8>},
                                     {attn_sweep_kernel<false, 4>, attn_sweep_kernel<true, 4>},
                                     {attn_sweep_kernel<false, 2>, attn_sweep_kernel<true, 2>}};
  const int lds = 4 * 16384;        // three ring slots and the global token's rows; the redo gives each wave a slot
  const int wi = d.block == 8 ? 0 : (d.block == 4 ? 1 : 2);
  const int ei = (d.grid_h % 8 == 0 && d.grid_w % 8 == 0) ? 0 : 1;
  const ns_status rs = reserve_lds_once(reinterpret_cast<const void *>(kerns[wi][ei]), lds);
  if (rs != NS_OK) return rs;
  hipLaunchKernelGGL(kerns[wi][ei], dim3((unsigned)strips), dim3(256), lds, a.stream, p);
  return check_launch("attn_sweep_kernel");
}

}  // namespace ns
