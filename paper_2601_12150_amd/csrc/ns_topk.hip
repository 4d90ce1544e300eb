// Ranking and compaction (paper, "Time-Efficiency Optimization": rank the tokens by
// importance, discard the lowest-scoring proportion, shorten the sequence).
//
// Exact k-th largest score on an order-preserving integer image of the floats, then an
// in-index-order compaction, so the kept indices come out ascending and exact ties resolve to
// the lower index.
//   topk_select_reg_kernel: rows of up to 32768 scores, one workgroup of 16 waves per image, keys
//     in registers, 8-bit digit passes (radix select) until at most 1024 candidates are left, which
//     are ranked against each other: latency-bound, a score row is 64 - 128 KB.
//   topk_digit_pass_kernel / topk_place_kernel: longer rows, several
//     workgroups per image, four 8-bit digit passes (radix select), one launch each.
// gather_rows_kernel: copies the kept token rows (and the global rows) with 16-byte accesses.
#include "ns_common.h"

namespace ns {

namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// larger float <=> larger key; -0.0 and +0.0 map to the same key
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Adds the digits of the wave's candidate lanes to the wave's histogram.  Clustered scores put
// most lanes of a wave into the same few bins, where one LDS atomic per lane would serialise;
// so the first bins are peeled off with one add of a lane count each, and only what is left
// (digits that are spread out, hence rarely colliding) goes through per-lane atomics.
__device__ __forceinline__ void wave_histogram_add(uint32_t *h, bool cand, uint32_t digit, int lane) {
  unsigned long long rem = __ballot(cand);
#pragma unroll 1
  for (int it = 0; it < 2 && rem; it++) {
    const int leader = __ffsll((long long)rem) - 1;
    const uint32_t d0 = (uint32_t)__builtin_amdgcn_readlane((int)digit, leader);
    const unsigned long long same = __ballot(cand && digit == d0) & rem;
    if (lane == leader) atomicAdd(&h[d0], (uint32_t)__popcll(same));
    rem &= ~same;
  }
  if ((rem >> lane) & 1ull) atomicAdd(&h[digit], 1u);
}

// Sums inside a wave without a trip through LDS: DPP row shifts add up the 16 lanes of a row, the
// four row totals travel through scalar registers.
// Inclusive prefix sum over the lanes of a wave (lane l: x of lanes 0..l).
__device__ __forceinline__ uint32_t wave_prefix_incl(uint32_t x, int lane) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);   // row_shr:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);
  const uint32_t r0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15), r1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31),
                 r2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
  const int row = lane >> 4;
  return x + (row > 0 ? r0 : 0u) + (row > 1 ? r1 : 0u) + (row > 2 ? r2 : 0u);
}
// Inclusive suffix sum (lane l: x of lanes l..63).
__device__ __forceinline__ uint32_t wave_suffix_incl(uint32_t x, int lane) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x101, 0xf, 0xf, true);   // row_shl:1
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x102, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x104, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x108, 0xf, 0xf, true);
  const uint32_t r1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 16), r2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 32),
                 r3 = (uint32_t)__builtin_amdgcn_readlane((int)x, 48);
  const int row = lane >> 4;
  return x + (row < 1 ? r1 : 0u) + (row < 2 ? r2 : 0u) + (row < 3 ? r3 : 0u);
}
// Sum of x over lanes 0..15 (one DPP row), the same in every lane.
__device__ __forceinline__ uint32_t row0_total(uint32_t x) {
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);
  x += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);
  return (uint32_t)__builtin_amdgcn_readlane((int)x, 15);
}

// Threads 0..255 bring the number of candidates per digit; sel[0] = the digit that holds the
// need-th largest candidate, sel[1] = how many keys of that digit are still needed, sel[2] = how
// many candidates that digit holds.
__device__ __forceinline__ void choose_digit(uint32_t tot, uint32_t need, int tid, int wave, int lane,
                                             uint32_t *wtot, uint32_t *sel) {
  uint32_t above = 0;
  if (tid < 256) {
    const uint32_t incl = wave_suffix_incl(tot, lane);   // lanes >= lane
    if (lane == 0) wtot[wave] = incl;
    above = incl - tot;
  }
  __syncthreads();
  if (tid < 256) {
    for (int w = wave + 1; w < 4; w++) above += wtot[w];
    if (above < need && need <= above + tot) {   // exactly one digit satisfies this
      sel[0] = (uint32_t)tid;
      sel[1] = need - above;
      sel[2] = tot;
    }
  }
  __syncthreads();
}

constexpr int kDirectMax = 1024;   // candidates that the direct ranking below takes: one per thread

// Rows of N <= 1024 * KPT scores, one workgroup per image, every key in a register: the selection
// and the compaction read global memory exactly once.  Wave w owns the 64*KPT consecutive indices
// from w*64*KPT; in its group i (256 indices) lane l holds the four indices 256*i + 4*l .. + 3.
// So a wave loads 1 KB of consecutive scores per instruction, index order is (wave, group, lane,
// element), and the kept indices of a group go to consecutive output positions in lane order.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void topk_select_reg_kernel(const float *scores, int N, int k,
                                                                      const int32_t *coords_in,
                                                                      int32_t *kept,
                                                                      int32_t *coords_out) {
  static_assert(KPT % 4 == 0, "keys are held in groups of four");
  const int b = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *sc = scores + (size_t)b * N;
  __shared__ __attribute__((aligned(16))) uint32_t hist[256 * 32];
  __shared__ uint32_t wsum[4], sel[3], ncand;
  __shared__ uint32_t wgt[kSelWaves], weq[kSelWaves];

  // Padding slots hold key 0.  A real key is never 0 (that would be a NaN bit pattern), and
  // tau, the k-th largest real key, is therefore > 0: padding never passes "> tau" or "== tau".
  uint32_t key[KPT];
  const int j0 = wave * (64 * KPT) + 4 * lane;       // index of key[4*i + e]: j0 + 256*i + e
  const bool vec = (reinterpret_cast<uintptr_t>(sc) & 15) == 0;
#pragma unroll
  for (int i = 0; i < KPT / 4; i++) {
    const int j = j0 + 256 * i;
    if (vec && j + 4 <= N) {
      const f32x4 x = *reinterpret_cast<const f32x4 *>(sc + j);
#pragma unroll
      for (int e = 0; e < 4; e++) key[4 * i + e] = order_key(x[e]);
    } else {
#pragma unroll
      for (int e = 0; e < 4; e++) key[4 * i + e] = j + e < N ? order_key(sc[j + e]) : 0u;
    }
  }
  if (tid == 0) ncand = 0;
  // k-th largest key by 8-bit digit passes, most significant digit first (radix select): a pass
  // histograms the digit of the keys that match the prefix chosen so far, and the digit that holds
  // the left-th largest candidate extends the prefix.  The histogram is kept in 32 copies, bin d of
  // copy c at word 32*d + c, and lane l adds to copy l % 32: scores that cluster (most keys of a
  // wave in one bin) then still spread over 32 LDS banks instead of serialising on one address, so
  // a pass costs the same whatever the scores look like.  Once the candidates are few enough (after
  // two digits, as a rule), they are ranked against each other directly instead.
  // In the end `left` is the number of keys equal to tau that are kept.
  uint32_t tau = 0, left = (uint32_t)k;
  uint4 *hist4 = reinterpret_cast<uint4 *>(hist);
  for (int pass = 0; pass < 4; pass++) {
    const uint32_t mask = pass ? 0xffffffffu << (32 - 8 * pass) : 0u;
    if (pass > 0 && sel[2] <= (uint32_t)kDirectMax) {
      // ---- the candidates (keys that match the prefix) into a list, in any order: one atomic
      // per wave reserves the places of the wave's candidates
      uint32_t *cand = hist;
      __syncthreads();                       // everybody has read sel
      cand[tid] = 0u;                        // (a key 0 is below every real key)
      uint32_t m = 0;
#pragma unroll
      for (int i = 0; i < KPT; i++) m += key[i] != 0u && (key[i] & mask) == tau;
      const uint32_t incl = wave_prefix_incl(m, lane);
      const uint32_t wave_m = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
      __syncthreads();
      if (wave_m) {                          // (uniform in the wave)
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(&ncand, wave_m);
        uint32_t at = (uint32_t)__builtin_amdgcn_readlane((int)base, 0) + incl - m;
        if (m) {
#pragma unroll
          for (int i = 0; i < KPT; i++)
            if (key[i] != 0u && (key[i] & mask) == tau) cand[at++] = key[i];
        }
      }
      __syncthreads();
      // thread t ranks candidate t: tau is the candidate with fewer than `left` candidates above it
      // and at least `left` candidates not below it (equal candidates all say the same)
      // (waves without a candidate have nothing to do: the list is short)
      const uint32_t nc = ncand;
      if ((uint32_t)(tid & ~63) < nc) {
        const uint32_t n4 = (nc + 3u) >> 2, mine = cand[tid];
        uint32_t gt = 0, ge = 0;
        for (uint32_t c = 0; c < n4; c++) {
          const uint4 o = hist4[c];
          gt += (o.x > mine) + (o.y > mine) + (o.z > mine) + (o.w > mine);
          ge += (o.x >= mine) + (o.y >= mine) + (o.z >= mine) + (o.w >= mine);
        }
        if (mine != 0u && gt < left && left <= ge) {
          sel[0] = mine;
          sel[1] = left - gt;
        }
      }
      __syncthreads();
      tau = sel[0];
      left = sel[1];
      break;
    }
    const int shift = 24 - 8 * pass;
    __syncthreads();                         // (sel and the previous pass's histogram have been read)
    hist4[tid] = make_uint4(0u, 0u, 0u, 0u);
    hist4[tid + kSelThreads] = make_uint4(0u, 0u, 0u, 0u);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KPT; i++)
      if (key[i] != 0u && (key[i] & mask) == tau) atomicAdd(&hist[(((key[i] >> shift) & 255u) << 5) + (lane & 31)], 1u);
    __syncthreads();
    uint32_t tot = 0;
    if (tid < 256) {
      // (four copies per read, group (c + tid) % 8 in round c: two lanes per bank group in every
      // quarter wave, which is what a 16-byte read costs anyway)
#pragma unroll
      for (int c = 0; c < 8; c++) {
        const uint4 h4 = hist4[(tid << 3) + ((c + tid) & 7)];
        tot += (h4.x + h4.y) + (h4.z + h4.w);
      }
    }
    choose_digit(tot, left, tid, wave, lane, wsum, sel);
    tau |= sel[0] << shift;
    left = sel[1];
  }
  // every score above tau is kept; of those equal to it, the first `need` in index order
  const uint32_t need = left;
  // keys above tau and equal to it in this wave: counted on the scalar unit from the compare masks
  {
    uint32_t wave_gt = 0, wave_eq = 0;
#pragma unroll
    for (int i = 0; i < KPT; i++) {
      wave_gt += (uint32_t)__popcll(__ballot(key[i] > tau));
      wave_eq += (uint32_t)__popcll(__ballot(key[i] == tau));
    }
    if (lane == 0) { wgt[wave] = wave_gt; weq[wave] = wave_eq; }
  }
  __syncthreads();
  const uint32_t og = lane < wave ? wgt[lane & (kSelWaves - 1)] : 0u, oe = lane < wave ? weq[lane & (kSelWaves - 1)] : 0u;
  uint32_t run_gt = row0_total(og), run_eq = row0_total(oe);   // in the waves before this one (wave < 16 lanes of row 0)
  int32_t *kb = kept + (size_t)b * k;
#pragma unroll
  for (int i = 0; i < KPT / 4; i++) {
    uint32_t c = 0;
#pragma unroll
    for (int e = 0; e < 4; e++) c += (uint32_t)(key[4 * i + e] > tau) + ((uint32_t)(key[4 * i + e] == tau) << 16);
    const uint32_t incl = wave_prefix_incl(c, lane);           // at most 256 per half
    const uint32_t group = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    uint32_t ngt = run_gt + ((incl - c) & 0xffffu), neq = run_eq + ((incl - c) >> 16);
#pragma unroll
    for (int e = 0; e < 4; e++) {
      const bool gt = key[4 * i + e] > tau, eq = key[4 * i + e] == tau;
      if (gt || (eq && neq < need)) {
        const uint32_t pos = ngt + min(neq, need);
        const int j = j0 + 256 * i + e;
        if (pos < (uint32_t)k) {   // always
          kb[pos] = j;
          if (coords_in) coords_out[(size_t)b * k + pos] = coords_in[(size_t)b * N + j];
        }
      }
      ngt += gt;
      neq += eq;
    }
    run_gt += group & 0xffffu;
    run_eq += group >> 16;
  }
}

// ---- several workgroups per image (score rows too long for one CU to select from quickly)
//
// Four digit passes of 8 bits over the order-preserving keys, most significant first, and a
// placement pass, each one launch over (chunks, images).  A pass histograms the digit of the keys
// that match the prefix chosen so far, per chunk, into `part`; the next launch begins by adding the
// chunks' histograms (every workgroup does so for itself: a few hundred loads) and choosing the
// digit that holds the k-th largest key.  No atomics on global memory, no waiting between
// workgroups: the launches order the passes.
struct SelState { uint32_t prefix, need; };

// The state after digit `upto` (0..3) has been chosen, from the state before and that digit's
// histograms; workgroup 0 of the image records it for the next launch.  The histograms were
// written by other workgroups (other L2s): every load is a long trip, so all threads take part
// (thread t: digit t % 256, every fourth chunk) and keep eight loads in flight.
// quarter[4..7], if asked for (before >= 0): the same sums over the chunks below `before` only.
__device__ __forceinline__ SelState advance_state(int upto, int b, int B, int k, int nchunk, const uint32_t *part,
                                                  SelState *state, bool record, int before, int tid, int wave,
                                                  int lane, uint32_t *wtot, uint32_t *sel, uint32_t (*quarter)[256]) {
  SelState st = {0u, (uint32_t)k};
  if (upto > 0) st = state[(size_t)(upto - 1) * B + b];
  {
    const uint32_t *h = part + ((size_t)upto * B + b) * (size_t)nchunk * 256 + (tid & 255);
    uint32_t acc = 0, acc_before = 0;
#pragma unroll 8
    for (int c = tid >> 8; c < nchunk; c += 4) {
      const uint32_t n = h[(size_t)c * 256];
      acc += n;
      acc_before += c < before ? n : 0u;
    }
    quarter[tid >> 8][tid & 255] = acc;
    if (before >= 0) quarter[4 + (tid >> 8)][tid & 255] = acc_before;
  }
  __syncthreads();
  const uint32_t tot = tid < 256 ? quarter[0][tid] + quarter[1][tid] + quarter[2][tid] + quarter[3][tid] : 0u;
  choose_digit(tot, st.need, tid, wave, lane, wtot, sel);
  st.prefix |= sel[0] << (24 - 8 * upto);
  st.need = sel[1];
  if (record && tid == 0) state[(size_t)upto * B + b] = st;
  return st;
}

// grid (nchunk, B): digit `pass` (0 = bits 31..24) of the keys of chunk blockIdx.x.  The last pass
// also counts the chunk's keys above the 24-bit prefix (they are kept whatever the last digit is).
__global__ __launch_bounds__(kSelThreads) void topk_digit_pass_kernel(const float *scores, int N, int k, int pass,
                                                                     int kpt, uint32_t *part, SelState *state,
                                                                     uint32_t *above) {
  const int b = blockIdx.y, B = gridDim.y, c = blockIdx.x, nchunk = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *sc = scores + (size_t)b * N;
  __shared__ uint32_t hist[kSelWaves][256];
  __shared__ uint32_t wtot[4], sel[3], wabove[kSelWaves];
  SelState st = {0u, (uint32_t)k};
  if (pass > 0)     // (the first rows of hist serve as its exchange buffer)
    st = advance_state(pass - 1, b, B, k, nchunk, part, state, c == 0, -1, tid, wave, lane, wtot, sel, hist);
  for (int i = tid; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
  __syncthreads();
  const uint32_t mask = pass ? 0xffffffffu << (32 - 8 * pass) : 0u;
  const int shift = 24 - 8 * pass;
  const int base = c * kpt * kSelThreads;
  uint32_t nabove = 0;     // wave-uniform
  for (int i = 0; i < kpt; i++) {
    const int j = base + i * kSelThreads + tid;
    bool cand = false, over = false;
    uint32_t digit = 0;
    if (j < N) {
      const uint32_t key = order_key(sc[j]);
      cand = (key & mask) == st.prefix;
      over = (key & mask) > st.prefix;
      digit = (key >> shift) & 255u;
    }
    wave_histogram_add(hist[wave], cand, digit, lane);
    if (pass == 3) nabove += (uint32_t)__popcll(__ballot(over));
  }
  if (pass == 3 && lane == 0) wabove[wave] = nabove;
  __syncthreads();
  if (tid < 256) {
    uint32_t tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; w++) tot += hist[w][tid];
    part[(((size_t)pass * B + b) * nchunk + c) * 256 + tid] = tot;
  }
  if (pass == 3 && tid == 0) {
    uint32_t t = 0;
    for (int w = 0; w < kSelWaves; w++) t += wabove[w];
    above[(size_t)b * nchunk + c] = t;
  }
}

// grid (nchunk, B): the kept keys of chunk blockIdx.x go to their places (ascending index order;
// of the keys equal to the k-th largest, the first `need` in index order are kept).  What the
// chunks before this one keep comes from their histograms of the last digit and their counts of
// keys above the prefix: no key of another chunk is read.
__global__ __launch_bounds__(kSelThreads) void topk_place_kernel(const float *scores, int N, int k, int kpt,
                                                                const uint32_t *part, SelState *state,
                                                                const uint32_t *above, const int32_t *coords_in,
                                                                int32_t *kept, int32_t *coords_out) {
  const int b = blockIdx.y, B = gridDim.y, c = blockIdx.x, nchunk = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *sc = scores + (size_t)b * N;
  __shared__ uint32_t quarter[8][256];
  __shared__ uint32_t wtot[4], sel[3];
  __shared__ uint32_t wgt[kSelWaves], weq[kSelWaves];
  const uint32_t above_mine = tid < c ? above[(size_t)b * nchunk + tid] : 0u;     // at most 128 chunks
  const SelState st = advance_state(3, b, B, k, nchunk, part, state, false, c, tid, wave, lane, wtot, sel, quarter);
  const uint32_t tau = st.prefix, need = st.need, digit = tau & 255u;
  uint32_t cgt = above_mine, ceq = 0;
  if (tid < 256) {
    const uint32_t n = quarter[4][tid] + quarter[5][tid] + quarter[6][tid] + quarter[7][tid];
    cgt += (uint32_t)tid > digit ? n : 0u;
    ceq = (uint32_t)tid == digit ? n : 0u;
  }
  if (wave < 4) {
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) {
      cgt += (uint32_t)__shfl_xor((int)cgt, sft);
      ceq += (uint32_t)__shfl_xor((int)ceq, sft);
    }
    if (lane == 0) { wgt[wave] = cgt; weq[wave] = ceq; }
  }
  __syncthreads();
  uint32_t gt_before = wgt[0] + wgt[1] + wgt[2] + wgt[3], eq_before = weq[0] + weq[1] + weq[2] + weq[3];
  __syncthreads();
  const int base = c * kpt * kSelThreads;
  int32_t *kb = kept + (size_t)b * k;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int i = 0; i < kpt; i++) {          // index order inside the chunk: (i, wave, lane)
    const int j = base + i * kSelThreads + tid;
    const uint32_t key = j < N ? order_key(sc[j]) : 0u;
    const bool gt = j < N && key > tau, eq = j < N && key == tau;
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    if (lane == 0) { wgt[wave] = (uint32_t)__popcll(bgt); weq[wave] = (uint32_t)__popcll(beq); }
    __syncthreads();
    uint32_t my_gt = gt_before + (uint32_t)__popcll(bgt & lt), my_eq = eq_before + (uint32_t)__popcll(beq & lt);
    uint32_t all_gt = 0, all_eq = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; w++) {
      my_gt += w < wave ? wgt[w] : 0u;
      my_eq += w < wave ? weq[w] : 0u;
      all_gt += wgt[w];
      all_eq += weq[w];
    }
    if (gt || (eq && my_eq < need)) {
      const uint32_t pos = my_gt + min(my_eq, need);
      if (pos < (uint32_t)k) {   // always, when the scores hold no NaN
        kb[pos] = j;
        if (coords_in) coords_out[(size_t)b * k + pos] = coords_in[(size_t)b * N + j];
      }
    }
    gt_before += all_gt;
    eq_before += all_eq;
    __syncthreads();
  }
}

// grid (ceil((G+k)/4), B), 256 threads: one wave per output row; the G global rows come first.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *x, const int32_t *kept,
                                                          uint4 *y, int N, int k, int G, int vec_per_row) {
  const int b = blockIdx.y;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= G + k) return;
  const int src = row < G ? row : G + kept[(size_t)b * k + row - G];
  const uint4 *xs = x + ((size_t)b * (G + N) + src) * vec_per_row;
  uint4 *yd = y + ((size_t)b * (G + k) + row) * vec_per_row;
  // (streamed once: non-temporal accesses leave the caches to the kernels around this one)
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const u32x4 *src4 = reinterpret_cast<const u32x4 *>(xs);
  u32x4 *dst4 = reinterpret_cast<u32x4 *>(yd);
  for (int i = lane; i < vec_per_row; i += 64) __builtin_nontemporal_store(__builtin_nontemporal_load(src4 + i), dst4 + i);
}

}  // namespace

// Keys per thread of the several-workgroup selection: at most 128 chunks per image.
static int multi_kpt(int N) { return (int)(((long long)N + 128LL * kSelThreads - 1) / (128LL * kSelThreads)); }
static int multi_chunks(int N) { return (N + multi_kpt(N) * kSelThreads - 1) / (multi_kpt(N) * kSelThreads); }

// Keys per thread of the one-workgroup selection at most.  (With 64 keys a row of 65536 scores takes one
// compute unit 43 us; the five launches of the several-workgroup selection take 26 us plus their gaps.)
constexpr int kRegMaxKeys = 32;

size_t topk_select_workspace_bytes(int B, int N) {
  if (N <= kRegMaxKeys * kSelThreads) return 0;                    // one workgroup per image, state in registers and LDS
  return (size_t)4 * B * multi_chunks(N) * 256 * sizeof(uint32_t) + (size_t)4 * B * sizeof(SelState) +
         (size_t)B * multi_chunks(N) * sizeof(uint32_t);
}

ns_status launch_topk_select(int B, int N, int k, const float *scores, const int32_t *coords_in,
                             int32_t *kept, int32_t *coords_out, void *ws, hipStream_t s) {
  if (N <= kRegMaxKeys * kSelThreads) {
    const dim3 grid(B), block(kSelThreads);
    if (N <= 4 * kSelThreads)
      hipLaunchKernelGGL(topk_select_reg_kernel<4>, grid, block, 0, s, scores, N, k, coords_in, kept, coords_out);
    else if (N <= 8 * kSelThreads)
      hipLaunchKernelGGL(topk_select_reg_kernel<8>, grid, block, 0, s, scores, N, k, coords_in, kept, coords_out);
    else if (N <= 16 * kSelThreads)
      hipLaunchKernelGGL(topk_select_reg_kernel<16>, grid, block, 0, s, scores, N, k, coords_in, kept, coords_out);
    else
      hipLaunchKernelGGL(topk_select_reg_kernel<32>, grid, block, 0, s, scores, N, k, coords_in, kept, coords_out);
    return check_launch("topk_select_reg_kernel");
  }
  const int kpt = multi_kpt(N), nchunk = multi_chunks(N);
  uint32_t *part = static_cast<uint32_t *>(ws);
  SelState *state = reinterpret_cast<SelState *>(part + (size_t)4 * B * nchunk * 256);
  uint32_t *above = reinterpret_cast<uint32_t *>(state + (size_t)4 * B);
  for (int pass = 0; pass < 4; pass++)
    hipLaunchKernelGGL(topk_digit_pass_kernel, dim3(nchunk, B), dim3(kSelThreads), 0, s, scores, N, k, pass, kpt,
                       part, state, above);
  hipLaunchKernelGGL(topk_place_kernel, dim3(nchunk, B), dim3(kSelThreads), 0, s, scores, N, k, kpt, part, state,
                     above, coords_in, kept, coords_out);
  return check_launch("topk_place_kernel");
}

ns_status launch_gather_rows(int B, int N, int k, int G, size_t row_bytes, const void *x,
                             const int32_t *kept, void *y, hipStream_t s) {
  dim3 grid((G + k + 3) / 4, B);
  hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(256), 0, s, static_cast<const uint4 *>(x), kept,
                     static_cast<uint4 *>(y), N, k, G, (int)(row_bytes / 16));
  return check_launch("gather_rows_kernel");
}

}  // namespace ns
