// Exact k-th-largest selection and order-preserving compaction over the pages of one
// (sequence, query head), shared by the top-k and the Gaussian-aware selectors.
// One 1024-thread workgroup; keys are order-preserving uint32 images of float scores.
#pragma once
#include "ekv_device.h"

namespace ekv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kDigitBits = 11;
constexpr int kBins = 1 << kDigitBits;

struct SelectShared {
  uint32_t hist[kBins];
  int scan_buf[kSelWaves + 1];
  uint32_t red_u[kSelWaves];
  uint32_t digit, above;
};

// Exclusive prefix sum over the block in thread order; `total` receives the block sum.
// Contains barriers: all threads must call it.
__device__ __forceinline__ int block_excl_scan(int v, int* buf, int& total) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int inc = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const int t = __shfl_up(inc, d);
    if (lane >= d) inc += t;
  }
  __syncthreads();
  if (lane == 63) buf[w] = inc;
  __syncthreads();
  int base = 0, tot = 0;
  for (int i = 0; i < kSelWaves; ++i) {
    const int c = buf[i];
    if (i < w) base += c;
    tot += c;
  }
  total = tot;
  return base + inc - v;
}

// Finds the k-th largest key among keyfn(0..M-1) (1 <= k <= M) by radix selection on (key - min key),
// 11 bits per pass over only as many bits as the key range needs.  Returns kmin (the smallest key),
// vT = (k-th largest key) - kmin, and k_eq = how many elements equal to it belong to the top k.
template <typename KeyFn>
__device__ __forceinline__ void radix_select_kth(KeyFn keyfn, int M, int k, SelectShared& sh,
                                                 uint32_t& kmin_out, uint32_t& vT_out, int& k_eq_out) {
  const int tid = threadIdx.x;
  uint32_t lo = 0xffffffffu, hi = 0u;
  for (int p = tid; p < M; p += kSelThreads) {
    const uint32_t key = keyfn(p);
    lo = min(lo, key); hi = max(hi, key);
  }
  for (int d = 32; d >= 1; d >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, d));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, d));
  }
  __syncthreads();
  if ((tid & 63) == 0) sh.red_u[tid >> 6] = lo;
  __syncthreads();
  for (int i = 0; i < kSelWaves; ++i) lo = min(lo, sh.red_u[i]);
  __syncthreads();
  if ((tid & 63) == 0) sh.red_u[tid >> 6] = hi;
  __syncthreads();
  for (int i = 0; i < kSelWaves; ++i) hi = max(hi, sh.red_u[i]);
  const uint32_t kmin = lo;
  const uint32_t range = hi - lo;
  int shift = range ? 32 - __clz(range) : 0;     // significant bits of (key - kmin)

  uint32_t prefix = 0;       // high bits of the answer fixed so far: (v >> shift) == prefix
  int k_rem = k;             // rank of the answer among the elements sharing that prefix
  while (shift > 0) {
    const int dbits = min(kDigitBits, shift);
    shift -= dbits;
    const uint32_t dmask = (1u << dbits) - 1u;
    __syncthreads();
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    __syncthreads();
    for (int p = tid; p < M; p += kSelThreads) {
      const uint32_t v = keyfn(p) - kmin;
      if ((uint32_t)((uint64_t)v >> (shift + dbits)) == prefix) atomicAdd(&sh.hist[(v >> shift) & dmask], 1u);
    }
    __syncthreads();
    // thread t owns digits (kBins-1-2t) and (kBins-2-2t): scan from the top digit downwards
    const int d_hi = kBins - 1 - 2 * tid, d_lo = d_hi - 1;
    const int c_hi = (int)sh.hist[d_hi], c_lo = (int)sh.hist[d_lo];
    int total;
    const int above = block_excl_scan(c_hi + c_lo, sh.scan_buf, total);
    if (above < k_rem && k_rem <= above + c_hi) { sh.digit = d_hi; sh.above = above; }
    else if (above + c_hi < k_rem && k_rem <= above + c_hi + c_lo) { sh.digit = d_lo; sh.above = above + c_hi; }
    __syncthreads();
    prefix = (prefix << dbits) | sh.digit;
    k_rem -= (int)sh.above;
  }
  kmin_out = kmin; vT_out = prefix; k_eq_out = k_rem;
}

// Writes, in ascending page order, every page whose v = keyfn(p) - kmin exceeds vT, plus the first
// k_eq pages (by index) with v == vT.  Thread t owns the contiguous page range [t*ipt, (t+1)*ipt).
template <typename KeyFn>
__device__ __forceinline__ void compact_ordered(KeyFn keyfn, int M, uint32_t kmin, uint32_t vT, int k_eq,
                                                SelectShared& sh, int32_t* __restrict__ out) {
  const int tid = threadIdx.x;
  const int ipt = (M + kSelThreads - 1) / kSelThreads;
  const int p0 = min(tid * ipt, M), p1 = min(p0 + ipt, M);
  int n_gt = 0, n_eq = 0;
  for (int p = p0; p < p1; ++p) {
    const uint32_t v = keyfn(p) - kmin;
    n_gt += v > vT; n_eq += v == vT;
  }
  int tot_gt, tot_eq;
  const int gt_before = block_excl_scan(n_gt, sh.scan_buf, tot_gt);
  const int eq_before = block_excl_scan(n_eq, sh.scan_buf, tot_eq);
  int eq_rank = eq_before;
  int o = gt_before + min(eq_before, k_eq);
  for (int p = p0; p < p1; ++p) {
    const uint32_t v = keyfn(p) - kmin;
    bool take = v > vT;
    if (v == vT) { take = eq_rank < k_eq; ++eq_rank; }
    if (take) out[o++] = p;
  }
}

}  // namespace ekv
