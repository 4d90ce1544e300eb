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
      const unsigned long long act = __ballot(cand);
      if (act) {
        // clustered scores put whole waves into one bin: count those with a single add
        const int leader = __ffsll((long long)act) - 1;
        const uint32_t d0 = __shfl(digit, leader);
        const unsigned long long same = __ballot(cand && digit == d0);
        if (same == act) {
          if (lane == leader) atomicAdd(&hist[wave][d0], (uint32_t)__popcll(act));
        } else if (cand) {
          atomicAdd(&hist[wave][digit], 1u);
        }
      }
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

// grid (ceil((1+k)/4), B), 256 threads: one wave per output row.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint4 *x, const int32_t *kept,
                                                          uint4 *y, int N, int k, int vec_per_row) {
  const int b = blockIdx.y;
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row > k) return;
  const int src = row == 0 ? 0 : 1 + kept[(size_t)b * k + row - 1];
  const uint4 *xs = x + ((size_t)b * (1 + N) + src) * vec_per_row;
  uint4 *yd = y + ((size_t)b * (1 + k) + row) * vec_per_row;
  for (int i = lane; i < vec_per_row; i += 64) yd[i] = xs[i];
}

}  // namespace

ns_status launch_topk_select(int B, int N, int k, const float *scores, const int32_t *coords_in,
                             int32_t *kept, int32_t *coords_out, hipStream_t s) {
  hipLaunchKernelGGL(topk_select_kernel, dim3(B), dim3(kSelThreads), 0, s, scores, N, k, coords_in,
                     kept, coords_out);
  return check_launch("topk_select_kernel");
}

ns_status launch_gather_rows(int B, int N, int k, size_t row_bytes, const void *x,
                             const int32_t *kept, void *y, hipStream_t s) {
  dim3 grid((1 + k + 3) / 4, B);
  hipLaunchKernelGGL(gather_rows_kernel, grid, dim3(256), 0, s, static_cast<const uint4 *>(x), kept,
                     static_cast<uint4 *>(y), N, k, (int)(row_bytes / 16));
  return check_launch("gather_rows_kernel");
}

}  // namespace ns
