// bf16 MFMA GEMM with a 256 x 256 workgroup tile for the linear maps of the transformer block
// (QKV, attention projection, MLP): C[m][n] = sum_k A[m][k] W[n][k] + bias[n], optional exact
// GELU, optional residual R[m][n].  A, W, R, C bf16 row-major, bias fp32, fp32 accumulation.
// Bound: bf16 MFMA, 2*M*N*K FLOP.
//
// Why this shape.  A wave that owns a 64x64 piece of the output reads 1 KB of fragments from LDS
// per v_mfma_f32_32x32x16_bf16, which is exactly the LDS bandwidth of a CU at full MFMA rate; with
// a 128 x 128 piece per wave (4 x 4 MFMA tiles, 256 accumulator registers) it is half of that.
// So: 4 waves per workgroup, one per SIMD, each with up to 512 registers; 256 (n) x 256 (m) per
// workgroup; k in slices of 64 through two LDS stages filled by direct global -> LDS transfers
// (rows of 128 bytes: a transfer then uses whole cache lines, which moves the same bytes in 3/4 of
// the time that 64-byte rows take); the transfer of a slice is requested as soon as every wave has
// read the last fragments of the slice before the previous one, a whole slice of work ahead;
// fragments of the next 16-wide k-step are read from LDS while the 16 MFMAs of the current one
// execute.  The product is formed transposed (W rows as
// the A operand) as in the smaller kernel; the epilogue transposes each 32-token slab through
// LDS so that bias / GELU / residual / store work on 16-byte pieces of full output rows.
//
// Rows.  With M = 256 q + rem and 0 < rem <= 32 (a full-grid sequence: rem is the number of
// global tokens in the batch) the last row tile takes the extra rows as a ninth 32-row slab
// instead of opening a nearly empty tile row, which would cost a whole extra round on a launch
// that otherwise fills the chip exactly once; the slab's 8 MFMA tiles are shared out two per
// wave.  Any other remainder gets a tile of its own whose waves only compute the slabs that
// hold rows.  Where M / 256 row tiles leave many CUs without work in the last round (a pruned
// sequence: 39 x 4 tiles on 256 CUs), tiles of 192 rows (three slabs per wave) are used instead
// when that shortens the launch.
#include "ns_common.h"

namespace ns {

namespace {

struct Gemm256Params {
  const uint16_t *a, *w, *r;
  const float *bias;
  uint16_t *c;
  int M, N, K;
  int gelu;
  int ntn, ntm;      // tiles along n and m
  int extended;      // the last row tile has 288 rows
  int n256;          // the first n256 rows of tiles have 256 token rows, the others 192 (three slabs per wave):
                     // the mix that fills the chip's rounds of workgroups best
};

constexpr int kStageW = 256 * 128;           // bytes: 256 weight rows x 64 k
constexpr int kStageX = 288 * 128;           // 288 token rows x 64 k
constexpr int kStage = kStageW + kStageX;
constexpr int kStages = 2;
constexpr int kEpiRow = 528;                 // bytes per staged output row: 128 floats + 16 pad
constexpr int kEpiWave = 32 * kEpiRow;

typedef bf16x8 __attribute__((address_space(3))) *lds_bf16x8_ptr;



// Accumulators of NS weight slabs x one 32-token slab -> LDS (fp32, [token][32*NS n]) -> lanes that
// own 8 consecutive n of one token: + bias, GELU, + residual, one 16-byte store.
// Waiting for a load also waits for every older store (one in-order counter), so no load may
// follow a store here: the bias is waited for up front and the residual rows of all passes are
// requested before the first store.
template <int NS, bool GELU, bool RES>
__device__ __forceinline__ void gemm256_emit(const Gemm256Params &p, unsigned char *ebuf, const f32x16 *const (&slab)[NS],
                                             int mbase, int nbase, int lane) {
  constexpr int LPT = NS * 4;                 // lanes per token row
  constexpr int PASSES = LPT / 2, TPP = 64 / LPT;   // tokens per pass
  const int l32 = lane & 31, hh = lane >> 5;
  const int nl = 8 * (lane & (LPT - 1));
  const int ncol = nbase + nl;
  f32x4 b0 = *reinterpret_cast<const f32x4 *>(p.bias + ncol);
  f32x4 b1 = *reinterpret_cast<const f32x4 *>(p.bias + ncol + 4);
  uint4 res[RES ? PASSES : 1];
  if (RES) {
#pragma unroll
    for (int ps = 0; ps < PASSES; ps++) {
      const int m = min(mbase + TPP * ps + lane / LPT, p.M - 1);
      res[ps] = *reinterpret_cast<const uint4 *>(p.r + (size_t)m * p.N + ncol);
    }
  }
#pragma unroll
  for (int ti = 0; ti < NS; ti++)
#pragma unroll
    for (int g = 0; g < 4; g++) {
      const f32x16 &a = *slab[ti];
      const f32x4 v = {a[4 * g], a[4 * g + 1], a[4 * g + 2], a[4 * g + 3]};
      *reinterpret_cast<f32x4 *>(ebuf + l32 * kEpiRow + (32 * ti + 8 * g + 4 * hh) * 4) = v;
    }
  asm volatile("" : "+v"(b0), "+v"(b1));      // the bias has arrived before the first store is issued
  auto pass = [&](int ps, const uint4 &r4) {
    const int t = TPP * ps + lane / LPT;
    const int m = mbase + t;
    const f32x4 v0 = *reinterpret_cast<const f32x4 *>(ebuf + t * kEpiRow + nl * 4);
    const f32x4 v1 = *reinterpret_cast<const f32x4 *>(ebuf + t * kEpiRow + nl * 4 + 16);
    float o[8] = {v0[0] + b0[0], v0[1] + b0[1], v0[2] + b0[2], v0[3] + b0[3],
                  v1[0] + b1[0], v1[1] + b1[1], v1[2] + b1[2], v1[3] + b1[3]};
    if (GELU) gelu_erf8(o);
    if (RES) {
      o[0] += bf16_lo(r4.x); o[1] += bf16_hi(r4.x); o[2] += bf16_lo(r4.y); o[3] += bf16_hi(r4.y);
      o[4] += bf16_lo(r4.z); o[5] += bf16_hi(r4.z); o[6] += bf16_lo(r4.w); o[7] += bf16_hi(r4.w);
    }
    if (m < p.M) {
      const uint4 u = {pack_bf16(o[0], o[1]), pack_bf16(o[2], o[3]), pack_bf16(o[4], o[5]), pack_bf16(o[6], o[7])};
      *reinterpret_cast<uint4 *>(p.c + (size_t)m * p.N + ncol) = u;
    }
  };
  if (RES) {
#pragma unroll
    for (int ps = 0; ps < PASSES; ps++) pass(ps, res[ps]);
  } else {
#pragma unroll 2
    for (int ps = 0; ps < PASSES; ps++) pass(ps, res[0]);
  }
}

// One wave's work on one workgroup tile.  NTJ: 32-row token slabs of its own 128 rows that this
// wave computes (0..4).  EXT: the tile has a ninth token slab (rows 256..287); this wave then
// also computes that slab against weight slabs 2*WM and 2*WM+1 of its n half, and every wave
// issues 9 instead of 8 token-row requests per k-slice.
template <int NTJ, bool EXT, int WM, bool GELU, bool RES, int TM = 256>
__device__ __forceinline__ void gemm256_wave(const Gemm256Params &p, unsigned char *smem, int m0, int n0,
                                             int wave, int lane) {
  static_assert(TM == 256 || (TM == 192 && !EXT && NTJ <= 3), "192-row tiles: three slabs per wave, no ninth slab");
  constexpr int NT = NTJ > 0 ? NTJ : 1;
  constexpr int XREQ = EXT ? 9 : TM / 32;    // requests of 8 token rows per wave
  constexpr int WROWS = TM / 2;              // token rows per pair of waves
  const int l32 = lane & 31, hh = lane >> 5;
  const int wm = wave >> 1, wn = wave & 1;
  const uint32_t lds0 = (uint32_t)(size_t)((__attribute__((address_space(3))) unsigned char *)smem);
  const uint32_t rowB = (uint32_t)p.K * 2u;
  const char *ab = reinterpret_cast<const char *>(p.a);
  const char *wb = reinterpret_cast<const char *>(p.w);

  // ---- transfers.  A request moves 8 rows x 128 bytes: slot `lane` is row lane/8, physical
  // 16-byte chunk lane%8, which holds logical chunk (lane%8) ^ ((row >> 1) & 7), row counted
  // within the stage.  (The LDS has 64 banks and serves 16 lanes of a 16-byte read per clock: two
  // rows of 128 bytes span the banks once, so rows 2j and 2j+1 share a swizzle and the 16 rows
  // that 16 consecutive lanes read land on 16 different bank groups.)  Requests start at
  // multiples of 8 rows, so (row >> 1) & 7 = 4 * (request & 1) + lane/16.
  const int drow = lane >> 3;
  auto dchunk = [&](int req) { return 16u * ((lane & 7) ^ ((4 * (req & 1) + (drow >> 1)) & 7)); };
  const int wreq0 = wave * 8;                                        // weight requests: 8 per wave
  const int xreq0 = wave * XREQ;                                     // token requests
  const uint32_t woff[2] = {(uint32_t)(n0 + wreq0 * 8 + drow) * rowB + dchunk(0),
                            (uint32_t)(n0 + wreq0 * 8 + drow) * rowB + dchunk(1)};
  uint32_t xoff[XREQ];
#pragma unroll
  for (int j = 0; j < XREQ; j++) {
    const int m = min(m0 + (xreq0 + j) * 8 + drow, p.M - 1);         // rows past M repeat the last row
    xoff[j] = (uint32_t)m * rowB + dchunk(xreq0 + j);
  }
  auto issue = [&](int kt, int stage) {
    const char *ak = ab + (size_t)kt * 128, *wk = wb + (size_t)kt * 128;
    const uint32_t base = lds0 + stage * kStage;
#pragma unroll
    for (int j = 0; j < 8; j++) dma16(wk + (size_t)j * 8 * rowB, woff[j & 1], base + (wreq0 + j) * 1024);
#pragma unroll
    for (int j = 0; j < XREQ; j++) dma16(ak, xoff[j], base + kStageW + (xreq0 + j) * 1024);
  };
  constexpr int PER_SLICE = 8 + XREQ;

  // ---- fragment reads: lane (row l32 of a 32-row slab, half hh) reads logical chunk 2*ks + hh of
  // k-step ks = 0..3, i.e. physical chunk (2*ks + hh) ^ ((l32 >> 1) & 7) (slabs start at multiples of 32 rows)
  unsigned char *wrd[4], *xrd[4], *erd[4];
#pragma unroll
  for (int ks = 0; ks < 4; ks++) {
    const int ch = 16 * ((2 * ks + hh) ^ ((l32 >> 1) & 7));
    wrd[ks] = smem + (wn * 128 + l32) * 128 + ch;
    xrd[ks] = smem + kStageW + (wm * WROWS + l32) * 128 + ch;
    erd[ks] = smem + kStageW + (256 + l32) * 128 + ch;
  }
  bf16x8 fw[2][4], fx[2][NT], fe[2];
  auto read_frags = [&](int buf, int stage, int ks) {
    const int so = stage * kStage;
#pragma unroll
    for (int ti = 0; ti < 4; ti++) fw[buf][ti] = *(lds_bf16x8_ptr)(wrd[ks] + so + ti * 4096);
#pragma unroll
    for (int tj = 0; tj < NTJ; tj++) fx[buf][tj] = *(lds_bf16x8_ptr)(xrd[ks] + so + tj * 4096);
    if (EXT) fe[buf] = *(lds_bf16x8_ptr)(erd[ks] + so);
  };
  f32x16 acc[4][NT];   // [weight slab][token slab]: register e = n 8*(e/4) + 4*hh + e%4, lane = token l32
#pragma unroll
  for (int ti = 0; ti < 4; ti++)
#pragma unroll
    for (int tj = 0; tj < NT; tj++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[ti][tj][e] = 0.f;
  f32x16 acce[2];      // ninth token slab x weight slabs 2*WM, 2*WM+1
#pragma unroll
  for (int e = 0; e < 16; e++) { acce[0][e] = 0.f; acce[1][e] = 0.f; }
  auto mma = [&](int buf) {
#pragma unroll
    for (int ti = 0; ti < 4; ti++)
#pragma unroll
      for (int tj = 0; tj < NTJ; tj++)
        acc[ti][tj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[buf][ti], fx[buf][tj], acc[ti][tj], 0, 0, 0);
    if (EXT) {
      // The compiler keeps every accumulator of its own MFMAs in the 256 accumulator registers;
      // 18 of them do not fit and would be rotated through moves in every iteration.  These two
      // are pinned to ordinary vector registers instead.  (Each is next touched 17 MFMAs later,
      // and read by other instructions only after the loop: no issue hazards to pad.)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acce[0]) : "v"(fw[buf][2 * WM]), "v"(fe[buf]));
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acce[1]) : "v"(fw[buf][2 * WM + 1]), "v"(fe[buf]));
    }
  };

  // Issue order of one k-step: the 16-byte LDS reads of the NEXT step's fragments are spread
  // between the MFMAs of the current one (one read per two MFMAs), so that neither the LDS
  // latency nor its transfer time is exposed.  Without this the scheduler sinks the reads below
  // the MFMAs that do not need them.
  auto interleave = [&]() {
#pragma unroll
    for (int i = 0; i < 4 + NTJ + (EXT ? 1 : 0); i++) {
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
      __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   // two MFMAs
    }
  };

  // ---- main loop over slices of 64.  At the top of iteration kt: slice kt has landed for every
  // wave, slice kt+1 is in flight into the other stage, fragment buffer 0 holds (slice kt, k-step
  // 0).  After the third k-step every wave has issued its last reads of slice kt; with the barrier
  // there slice kt+1 is complete for all, and slice kt+2 can be requested into slice kt's stage.
  const int nk = p.K / 64;
  issue(0, 0);
  if (nk > 1) {
    issue(1, 1);
    wait_vm<PER_SLICE>();
  } else {
    wait_vm<0>();
  }
  __syncthreads();
  read_frags(0, 0, 0);
  for (int kt = 0; kt < nk; kt++) {
    const int cur = kt & 1;
    read_frags(1, cur, 1);
    mma(0);
    interleave();
    read_frags(0, cur, 2);
    mma(1);
    interleave();
    read_frags(1, cur, 3);
    mma(0);
    interleave();
    wait_vm<0>();                                     // slice kt+1 (this wave's share)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the fragments of slice kt are in registers
    __syncthreads();
    if (kt + 2 < nk) issue(kt + 2, cur);
    read_frags(0, cur ^ 1, 0);
    mma(1);
    interleave();
  }
  __syncthreads();             // every wave is done with the stages: they become the epilogue's staging area

  // ---- epilogue, one 32-token slab at a time
  unsigned char *ebuf = smem + wave * kEpiWave;
#pragma unroll
  for (int tj = 0; tj < NTJ; tj++) {
    const f32x16 *const slab[4] = {&acc[0][tj], &acc[1][tj], &acc[2][tj], &acc[3][tj]};
    gemm256_emit<4, GELU, RES>(p, ebuf, slab, m0 + wm * WROWS + tj * 32, n0 + wn * 128, lane);
  }
  if (EXT) {
    const f32x16 *const slab[2] = {&acce[0], &acce[1]};
    gemm256_emit<2, GELU, RES>(p, ebuf, slab, m0 + 256, n0 + wn * 128 + 64 * WM, lane);
  }
}

template <bool GELU, bool RES>
__global__ __launch_bounds__(256) void gemm256_bf16_kernel(Gemm256Params p) {
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  // workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of tiles (n
  // fastest) so that the tiles sharing token rows and the weight matrix meet in one L2
  const int total = p.ntn * p.ntm;
  int bid = blockIdx.x;
  const bool uniform = p.n256 == 0 || p.n256 == p.ntm;     // (a mix of tile heights keeps the launch order: tall tiles first)
  if (uniform && total % 8 == 0) bid = (bid & 7) * (total / 8) + (bid >> 3);
  const int bm = bid / p.ntn, bn = bid - bm * p.ntn;
  const int tm = bm < p.n256 ? 256 : 192;
  const int m0 = bm < p.n256 ? bm * 256 : p.n256 * 256 + (bm - p.n256) * 192, n0 = bn * 256;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  const bool ext = p.extended && bm == p.ntm - 1;
  const int wm = wave >> 1;
  const int wrows = tm >> 1;
  const int rows = min(p.M - (m0 + wm * wrows), wrows);   // may be <= 0
  const int ntj = __builtin_amdgcn_readfirstlane(rows <= 0 ? 0 : (rows + 31) / 32);
  if (ext) {   // the extended tile is full: 256 + (1..32) rows
    if (wm) gemm256_wave<4, true, 1, GELU, RES>(p, smem, m0, n0, wave, lane);
    else gemm256_wave<4, true, 0, GELU, RES>(p, smem, m0, n0, wave, lane);
    return;
  }
  if (tm == 192) {
    switch (ntj) {
      case 3: gemm256_wave<3, false, 0, GELU, RES, 192>(p, smem, m0, n0, wave, lane); break;
      case 2: gemm256_wave<2, false, 0, GELU, RES, 192>(p, smem, m0, n0, wave, lane); break;
      case 1: gemm256_wave<1, false, 0, GELU, RES, 192>(p, smem, m0, n0, wave, lane); break;
      default: gemm256_wave<0, false, 0, GELU, RES, 192>(p, smem, m0, n0, wave, lane); break;
    }
    return;
  }
  switch (ntj) {
    case 4: gemm256_wave<4, false, 0, GELU, RES>(p, smem, m0, n0, wave, lane); break;
    case 3: gemm256_wave<3, false, 0, GELU, RES>(p, smem, m0, n0, wave, lane); break;
    case 2: gemm256_wave<2, false, 0, GELU, RES>(p, smem, m0, n0, wave, lane); break;
    case 1: gemm256_wave<1, false, 0, GELU, RES>(p, smem, m0, n0, wave, lane); break;
    default: gemm256_wave<0, false, 0, GELU, RES>(p, smem, m0, n0, wave, lane); break;
  }
}

}  // namespace

bool gemm256_supported(int M, int N, int K) {
  return M >= 256 && N % 256 == 0 && K % 64 == 0 && K >= 64;
}

ns_status launch_gemm256(const uint16_t *a, const uint16_t *w, const float *bias, const uint16_t *r,
                         uint16_t *c, int M, int N, int K, bool gelu, hipStream_t s) {
  if (!gemm256_supported(M, N, K)) return fail(NS_ERR_UNSUPPORTED, "GEMM shape M=%d N=%d K=%d", M, N, K);
  if ((long long)M * K * 2 >= 0x7fffffffLL || (long long)N * K * 2 >= 0x7fffffffLL)
    return fail(NS_ERR_UNSUPPORTED, "GEMM operand beyond 2 GiB");
  Gemm256Params p{a, w, r, bias, c, M, N, K, gelu ? 1 : 0, N / 256, 0, 0, 0};
  const int q = M / 256, rem = M % 256;
  p.extended = (rem > 0 && rem <= 32) ? 1 : 0;
  p.ntm = (rem == 0 || p.extended) ? q : q + 1;
  p.n256 = p.ntm;
  {
    // Rows of tiles: a of 256 token rows, then b of 192, a*256 + b*192 >= M.  Workgroups start in
    // launch order, a CU takes the next one when it is free: the mix with the shortest makespan
    // (a 192-row tile costs 0.8 of a 256-row one).
    const int cus = device_cu_count();
    auto makespan = [&](long long na, long long nb) -> double {
      // na*ntn tiles of cost 1.0, then nb*ntn of cost 0.8, each given to the unit that is free first.
      // After the tall tiles n2 units are free at t2 and the other n1 one tile time earlier, at t1.
      const long long ta = na * p.ntn;
      long long left = nb * p.ntn;
      const long long n2 = ta % cus, n1 = cus - n2;
      double t1 = (double)(ta / cus), t2 = t1 + 1.0;
      double end = n2 ? t2 : t1;
      while (left > 0) {
        if (n2 == 0 || t1 <= t2) {
          left -= std::min(left, n1);
          t1 += 0.8;
          end = std::max(end, t1);
        } else {
          left -= std::min(left, n2);
          t2 += 0.8;
          end = std::max(end, t2);
        }
      }
      return end;
    };
    double best = makespan(p.ntm, 0);    // (the ninth slab of an extended tile is not counted: it is cheap)
    int best_a = p.ntm, best_b = 0;
    const int max_b = (M + 191) / 192;
    for (int nb = 1; nb <= max_b; nb++) {
      const long long covered = (long long)nb * 192;
      const int na = covered >= M ? 0 : (int)((M - covered + 255) / 256);
      const double t = makespan(na, nb);
      if (t < best - 1e-9) { best = t; best_a = na; best_b = nb; }
    }
    if (best_b > 0) { p.n256 = best_a; p.ntm = best_a + best_b; p.extended = 0; }
  }
  const long long wgs = (long long)p.ntm * p.ntn;
  if (wgs > 0x7fffffffLL) return fail(NS_ERR_UNSUPPORTED, "GEMM grid too large");
  typedef void (*kern_t)(Gemm256Params);
  static const kern_t kerns[4] = {gemm256_bf16_kernel<false, false>, gemm256_bf16_kernel<false, true>,
                                  gemm256_bf16_kernel<true, false>, gemm256_bf16_kernel<true, true>};
  const ns_status rs = reserve_lds_once(reinterpret_cast<const void *>(kerns[(gelu ? 2 : 0) + (r ? 1 : 0)]), kStages * kStage);
  if (rs != NS_OK) return rs;
  hipLaunchKernelGGL(kerns[(gelu ? 2 : 0) + (r ? 1 : 0)], dim3((unsigned)wgs), dim3(256), kStages * kStage, s, p);
  return check_launch("gemm256_bf16_kernel");
}

}  // namespace ns
