// Ranking and compaction (paper, "Time-Efficiency Optimization": rank the tokens by
// importance, discard the lowest-scoring proportion, shorten the sequence).
//
// topk_select_kernel: exact k-th largest score by a 4-pass, 8-bit-digit radix select on an
// order-preserving integer image of the floats, then an in-index-order compaction, so the
// kept indices come out ascending and exact ties resolve to the lower index.  One workgroup
// of 16 waves per image: a score row is at most a few hundred KB, so the step is bound by
// latency, not by bandwidth.
// gather_rows_kernel: copies the kept token rows (and the CLS row) with 16-byte accesses.
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

__global__ __launch_bounds__(kSelThreads) void topk_select_kernel(const float *scores, int N, int k,
                                                                  const int32_t *coords_in,
                                                                  int32_t *kept,
                                                                  int32_t *coords_out) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *sc = scores + (size_t)b * N;
  __shared__ uint32_t hist[kSelWaves][256];
  __shared__ uint32_t wtot[4];
  __shared__ uint32_t s_prefix, s_need;
  __shared__ uint32_t wgt[kSelWaves], weq[kSelWaves];

  uint32_t prefix = 0, mask = 0, need = (uint32_t)k;
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = tid; i < kSelWaves * 256; i += kSelThreads) (&hist[0][0])[i] = 0;
    __syncthreads();
    for (int base = 0; base < N; base += kSelThreads) {
      const int j = base + tid;
      bool cand = false;
      uint32_t digit = 0;
      if (j < N) {
        const uint32_t key = order_key(sc[j]);
        cand = (key & mask) == prefix;
        digit = (key >> shift) & 255u;
      }
      wave_histogram_add(hist[wave], cand, digit, lane);
    }
    __syncthreads();
    // threads 0..255: bin totals, suffix sums (count of candidates with a larger digit)
    uint32_t tot = 0, above = 0;
    if (tid < 256) {
#pragma unroll
      for (int w = 0; w < kSelWaves; w++) tot += hist[w][tid];
      uint32_t incl = tot;   // inclusive suffix sum inside the wave: lanes >= lane
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const uint32_t t = __shfl_down(incl, off);
        if (lane + off < 64) incl += t;
      }
      if (lane == 0) wtot[wave] = incl;
      above = incl - tot;
    }
    __syncthreads();
    if (tid < 256) {
      for (int w = wave + 1; w < 4; w++) above += wtot[w];
      if (above < need && need <= above + tot) {   // exactly one bin satisfies this
        s_prefix = prefix | ((uint32_t)tid << shift);
        s_need = need - above;
      }
    }
    __syncthreads();
    prefix = s_prefix;
    need = s_need;
    mask |= 255u << shift;
    __syncthreads();
  }
  // prefix = key of the k-th largest score; `need` of the scores equal to it are kept (the
  // first ones in index order), all larger ones are kept.
  const uint32_t tau = prefix;
  const int per_wave = (N + kSelWaves - 1) / kSelWaves;
  const int lo = min(N, wave * per_wave), hi = min(N, lo + per_wave);
  uint32_t cgt = 0, ceq = 0;
  for (int base = lo; base < hi; base += 64) {
    const int j = base + lane;
    const uint32_t key = j < hi ? order_key(sc[j]) : 0u;
    cgt += (uint32_t)__popcll(__ballot(j < hi && key > tau));
    ceq += (uint32_t)__popcll(__ballot(j < hi && key == tau));
  }
  if (lane == 0) { wgt[wave] = cgt; weq[wave] = ceq; }
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; w++) { gt_before += wgt[w]; eq_before += weq[w]; }
  int32_t *kb = kept + (size_t)b * k;
  const unsigned long long lt = (1ull << lane) - 1ull;
  for (int base = lo; base < hi; base += 64) {
    const int j = base + lane;
    const uint32_t key = j < hi ? order_key(sc[j]) : 0u;
    const bool gt = j < hi && key > tau, eq = j < hi && key == tau;
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    const uint32_t my_gt = gt_before + (uint32_t)__popcll(bgt & lt);
    const uint32_t my_eq = eq_before + (uint32_t)__popcll(beq & lt);
    const bool take = gt || (eq && my_eq < need);
    if (take) {
      const uint32_t pos = my_gt + min(my_eq, need);
      kb[pos] = j;
      if (coords_in) coords_out[(size_t)b * k + pos] = coords_in[(size_t)b * N + j];
    }
    gt_before += (uint32_t)__popcll(bgt);
    eq_before += (uint32_t)__popcll(beq);
  }
}

// Register-resident variant for N <= 1024 * KPT: every thread keeps its KPT keys in registers
// (thread t holds indices i*1024 + t), so the selection and the compaction read global memory
// exactly once and the step is a few microseconds of ALU work.
template <int KPT>
__global__ __launch_bounds__(kSelThreads) void topk_select_reg_kernel(const float *scores, int N, int k,
                                                                      const int32_t *coords_in,
                                                                      int32_t *kept,
                                                                      int32_t *coords_out) {
  const int b = blockIdx.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const float *sc = scores + (size_t)b * N;
  __shared__ uint32_t wtot[2][kSelWaves];
  __shared__ uint32_t pgt[KPT * kSelWaves], peq[KPT * kSelWaves];   // per (i, wave) counts -> prefixes
  __shared__ uint32_t sgt[kSelWaves], seq[kSelWaves];

  // Padding slots hold key 0.  A real key is never 0 (that would be a NaN bit pattern), and
  // tau, the k-th largest real key, is therefore > 0: padding never passes "> tau" or "== tau".
  uint32_t key[KPT];
#pragma unroll
  for (int i = 0; i < KPT; i++) {
    const int j = i * kSelThreads + tid;
    key[i] = j < N ? order_key(sc[j]) : 0u;
  }
  // k-th largest key by bisection on its bits, most significant first: tau keeps a bit iff at
  // least k keys are >= the candidate.  A wave counts with one compare + one scalar popcount per
  // key slot (no LDS atomics, cost independent of how the scores cluster); the 16 wave counts
  // are exchanged through LDS, double-buffered so that one barrier per bit suffices.  (Measured:
  // the step time is set by the compares of all N keys on this one CU; two bits per step, with
  // three candidates, was slower.)
  auto block_total = [&](uint32_t wave_count, int slot) -> uint32_t {
    if (lane == 0) wtot[slot][wave] = wave_count;
    __syncthreads();
    uint32_t t = lane < kSelWaves ? wtot[slot][lane] : 0u;
    // sum over lanes 0..15 (one DPP row): row_shr 1, 2, 4, 8 leaves the total in lane 15
    t += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, 0x111, 0xf, 0xf, true);
    t += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, 0x112, 0xf, 0xf, true);
    t += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, 0x114, 0xf, 0xf, true);
    t += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)t, 0x118, 0xf, 0xf, true);
    return (uint32_t)__builtin_amdgcn_readlane((int)t, 15);
  };
  uint32_t tau = 0;
  int slot = 0;      // exchange buffer of the next block_total (they alternate)
  for (int bit = 31; bit >= 0; bit--) {
    const uint32_t cand = tau | (1u << bit);
    uint32_t c = 0;   // wave-uniform: lives in a scalar register
    if (KPT <= 16) {
#pragma unroll
      for (int i = 0; i < KPT; i++) c += (uint32_t)__popcll(__ballot(key[i] >= cand));   // padding keys are 0 < cand
    } else {
      // many keys per lane: count per lane on the vector ALU (compare + add with carry), one
      // reduction over the lanes per bit; the scalar unit, one per CU, is the bottleneck otherwise
      uint32_t cl = 0;
#pragma unroll
      for (int i = 0; i < KPT; i++) cl += key[i] >= cand ? 1u : 0u;
#pragma unroll
      for (int sft = 1; sft < 64; sft <<= 1) cl += (uint32_t)__shfl_xor((int)cl, sft);
      c = (uint32_t)__builtin_amdgcn_readfirstlane((int)cl);
    }
    const uint32_t tot = block_total(c, slot);
    slot ^= 1;
    if (tot >= (uint32_t)k) tau = cand;
    // exactly k keys are >= cand: they are the kept set, the remaining bits of the k-th key do
    // not matter (below, every key >= tau is then either above it or one of `need` equal ones)
    if (tot == (uint32_t)k) break;
  }
  uint32_t cg = 0;
#pragma unroll
  for (int i = 0; i < KPT; i++) cg += (uint32_t)__popcll(__ballot(key[i] > tau));
  // every score above tau is kept; of those equal to it, the first `need` in index order
  const uint32_t need = (uint32_t)k - block_total(cg, slot);
  // index order = (i, wave, lane); count per (i, wave), scan, then place
#pragma unroll
  for (int i = 0; i < KPT; i++) {
    const unsigned long long bgt = __ballot(key[i] > tau);
    const unsigned long long beq = __ballot(key[i] == tau);
    if (lane == 0) {
      pgt[i * kSelWaves + wave] = (uint32_t)__popcll(bgt);
      peq[i * kSelWaves + wave] = (uint32_t)__popcll(beq);
    }
  }
  __syncthreads();
  {
    // block-wide exclusive scan of the KPT*16 (<= 1024) counts: thread t owns entry t
    const bool own = tid < KPT * kSelWaves;
    const uint32_t g = own ? pgt[tid] : 0u, e = own ? peq[tid] : 0u;
    uint32_t ig = g, ie = e;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t tg = __shfl_up(ig, off), te = __shfl_up(ie, off);
      if (lane >= off) { ig += tg; ie += te; }
    }
    if (lane == 63) { sgt[wave] = ig; seq[wave] = ie; }
    __syncthreads();
    uint32_t bg = 0, be = 0;
    for (int w = 0; w < wave; w++) { bg += sgt[w]; be += seq[w]; }
    if (own) { pgt[tid] = bg + ig - g; peq[tid] = be + ie - e; }
    __syncthreads();
  }
  int32_t *kb = kept + (size_t)b * k;
  const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int i = 0; i < KPT; i++) {
    const int j = i * kSelThreads + tid;
    const bool gt = key[i] > tau, eq = key[i] == tau;
    const unsigned long long bgt = __ballot(gt), beq = __ballot(eq);
    const uint32_t my_gt = pgt[i * kSelWaves + wave] + (uint32_t)__popcll(bgt & lt);
    const uint32_t my_eq = peq[i * kSelWaves + wave] + (uint32_t)__popcll(beq & lt);
    if (gt || (eq && my_eq < need)) {
      const uint32_t pos = my_gt + min(my_eq, need);
      kb[pos] = j;
      if (coords_in) coords_out[(size_t)b * k + pos] = coords_in[(size_t)b * N + j];
    }
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
  for (int i = lane; i < vec_per_row; i += 64) yd[i] = xs[i];
}

}  // namespace

ns_status launch_topk_select(int B, int N, int k, const float *scores, const int32_t *coords_in,
                             int32_t *kept, int32_t *coords_out, hipStream_t s) {
  if (N <= 16 * kSelThreads)
    hipLaunchKernelGGL(topk_select_reg_kernel<16>, dim3(B), dim3(kSelThreads), 0, s, scores, N, k,
                       coords_in, kept, coords_out);
  else if (N <= 64 * kSelThreads)
    hipLaunchKernelGGL(topk_select_reg_kernel<64>, dim3(B), dim3(kSelThreads), 0, s, scores, N, k,
                       coords_in, kept, coords_out);
  else
    hipLaunchKernelGGL(topk_select_kernel, dim3(B), dim3(kSelThreads), 0, s, scores, N, k, coords_in,
                       kept, coords_out);
  return check_launch("topk_select_kernel");
}

ns_status launch_gather_rows(int B, int N, int k, int G, size_t row_bytes, const void *x,
                             const int32_t *kept, void *y, hipStream_t s) {
  dim3 grid((G + k + 3) / 4, B);
  hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(256), 0, s, static_cast<const uint4 *>(x), kept,
                     static_cast<uint4 *>(y), N, k, G, (int)(row_bytes / 16));
  return check_launch("gather_rows_kernel");
}

}  // namespace ns
