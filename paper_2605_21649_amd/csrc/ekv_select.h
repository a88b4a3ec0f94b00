// Exact k-th-largest selection and order-preserving compaction over the pages of one
// (sequence, query head), shared by the top-k and the Gaussian-aware selectors.
//
// One 1024-thread workgroup.  Keys are order-preserving uint32 images of float scores.  Wavefront w owns
// the contiguous page range [w*64*items, (w+1)*64*items) and lane l holds pages w*64*items + i*64 + l,
// i < items: loads are coalesced, keys can live in registers for all passes, and (w, i, l) order is
// ascending page order, so ballots give an ordered compaction without sorting.
#pragma once
#include "ekv_device.h"

namespace ekv {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;
constexpr int kDigitBits = 11;
constexpr int kBins = 1 << kDigitBits;
constexpr int kRankMax = 256;             // elements ranked directly once the radix passes have narrowed to so few

struct SelectShared {
  uint32_t hist[kBins];
  int scan_buf[kSelWaves + 1];
  uint32_t red_u[kSelWaves];
  int wave_gt[kSelWaves], wave_eq[kSelWaves];
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

// Keys of one (b,h) row.  ITEMS > 0: held in registers (M <= 1024*ITEMS); ITEMS == 0: recomputed from
// memory on every access (any M).  `fn(p)` gives the key of page p.  Slots past M hold the value 0.
// After rebase(kmin) every key is stored relative to kmin (so only one register array is live).
template <int ITEMS, typename KeyFn>
struct KeySet {
  KeyFn fn;
  int M, items, page0;                      // page0 = first page of this lane
  uint32_t base;                            // subtracted from every key
  uint32_t reg[ITEMS ? ITEMS : 1];
  __device__ __forceinline__ KeySet(KeyFn f, int M_) : fn(f), M(M_), base(0u) {
    items = ITEMS ? ITEMS : (M + kSelThreads - 1) / kSelThreads;
    page0 = (threadIdx.x >> 6) * 64 * items + (threadIdx.x & 63);
    if (ITEMS) {
      // unconditional loads from clamped pages (a load inside a divergent branch is waited for at
      // once, which would serialise all ITEMS loads), masked afterwards
#pragma unroll
      for (int i = 0; i < (ITEMS ? ITEMS : 1); ++i) reg[i] = fn(min(page(i), M - 1));
#pragma unroll
      for (int i = 0; i < (ITEMS ? ITEMS : 1); ++i) reg[i] = page(i) < M ? reg[i] : 0u;
    }
  }
  __device__ __forceinline__ int page(int i) const { return page0 + i * 64; }
  // before rebase(): slots past M hold 0 and no real key is 0 (checking the register instead of the page
  // index keeps the 128 page indices from being held in registers)
  __device__ __forceinline__ bool valid(int i) const { return ITEMS ? reg[i] != 0u : page(i) < M; }
  // key of slot i relative to `base`; slots past M (and keys below base) give 0
  __device__ __forceinline__ uint32_t key(int i) const {
    if (ITEMS) return reg[i];
    const uint32_t k0 = fn(min(page(i), M - 1));
    const uint32_t k = page(i) < M ? k0 : 0u;
    return max(k, base) - base;
  }
  // ITEMS == 0: the keys of slots i0 .. i0+7, all eight loads issued before any is used (a loop that calls
  // key(i) once per iteration waits for memory in every iteration).  Slots i >= items belong to the NEXT
  // wavefront's pages: the caller must skip them (i0 + j < items), not only pages >= M.
  __device__ __forceinline__ void key_batch(int i0, uint32_t (&k)[8]) const {
    uint32_t k0[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) k0[j] = fn(min(page(i0 + j), M - 1));
#pragma unroll
    for (int j = 0; j < 8; ++j) k[j] = max(page(i0 + j) < M ? k0[j] : 0u, base) - base;
  }
  __device__ __forceinline__ void rebase(uint32_t kmin) {
    base = kmin;
    if (ITEMS) {
#pragma unroll
      for (int i = 0; i < (ITEMS ? ITEMS : 1); ++i) reg[i] = max(reg[i], kmin) - kmin;
    }
  }
};

// Finds the k-th largest key (1 <= k <= M) by radix selection on (key - min key), 11 bits per pass over
// only as many bits as the key range needs.  Rebases the key set to the smallest valid key and returns
// vT = the k-th largest rebased key and k_eq = how many elements equal to it belong to the top k.
// Slots past M count as copies of the smallest key with the highest page indices, which never changes
// the answer for k <= M.
template <int ITEMS, typename KeyFn>
__device__ __forceinline__ void radix_select_kth(KeySet<ITEMS, KeyFn>& ks, int k, SelectShared& sh,
                                                 uint32_t& vT_out, int& k_eq_out) {
  const int tid = threadIdx.x;
  uint32_t lo = 0xffffffffu, hi = 0u;
  if constexpr (ITEMS == 0) {
    for (int i0 = 0; i0 < ks.items; i0 += 8) {
      uint32_t kb[8];
      ks.key_batch(i0, kb);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (i0 + j < ks.items && ks.page(i0 + j) < ks.M) { lo = min(lo, kb[j]); hi = max(hi, kb[j]); }
    }
  } else {
#pragma unroll
    for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) {
      if (ks.valid(i)) { const uint32_t key = ks.key(i); lo = min(lo, key); hi = max(hi, key); }
    }
  }
  for (int d = 32; d >= 1; d >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, d));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, d));
  }
  // both extremes in one exchange (the histogram array is free here: it is zeroed at the start of every pass)
  __syncthreads();
  if ((tid & 63) == 0) { sh.red_u[tid >> 6] = lo; sh.hist[tid >> 6] = hi; }
  __syncthreads();
  for (int i = 0; i < kSelWaves; ++i) { lo = min(lo, sh.red_u[i]); hi = max(hi, sh.hist[i]); }
  const uint32_t range = hi - lo;
  ks.rebase(lo);
  int shift = range ? 32 - __clz(range) : 0;     // significant bits of the rebased keys

  uint32_t prefix = 0;       // high bits of the answer fixed so far: (v >> shift) == prefix
  int k_rem = k;             // rank of the answer among the elements sharing that prefix
  const int n_pad = kSelThreads * (ITEMS ? ITEMS : ks.items) - ks.M;
  while (shift > 0) {
    const int dbits = min(kDigitBits, shift);
    shift -= dbits;
    const uint32_t dmask = (1u << dbits) - 1u;
    const int up = shift + dbits;                  // bits above the current digit: (v >> up) must equal prefix
    const bool first = up >= 32;                   // first pass of a full 32-bit range: every key matches
    const bool pad_counted = first || prefix == 0u;
    __syncthreads();
    for (int i = tid; i < kBins; i += kSelThreads) sh.hist[i] = 0;
    __syncthreads();
    // Slots past M hold the rebased key 0.  They are counted (as copies of the smallest key) but not sent
    // through the histogram one by one: thousands of atomics on one LDS address serialise.
    if constexpr (ITEMS == 0) {
      for (int i0 = 0; i0 < ks.items; i0 += 8) {
        uint32_t kb[8];
        ks.key_batch(i0, kb);
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (i0 + j < ks.items && ks.page(i0 + j) < ks.M && (first || (kb[j] >> up) == prefix))
            atomicAdd(&sh.hist[(kb[j] >> shift) & dmask], 1u);
      }
    } else {
#pragma unroll
      for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) {
        const uint32_t v = ks.key(i);
        if (ks.page(i) < ks.M && (first || (v >> up) == prefix)) atomicAdd(&sh.hist[(v >> shift) & dmask], 1u);
      }
    }
    if (tid == 0 && pad_counted && n_pad > 0) atomicAdd(&sh.hist[0], (uint32_t)n_pad);
    __syncthreads();
    // thread t owns digits (kBins-1-2t) and (kBins-2-2t): scan from the top digit downwards
    const int d_hi = kBins - 1 - 2 * tid, d_lo = d_hi - 1;
    const int c_hi = (int)sh.hist[d_hi], c_lo = (int)sh.hist[d_lo];
    int total;
    const int above = block_excl_scan(c_hi + c_lo, sh.scan_buf, total);
    if (above < k_rem && k_rem <= above + c_hi) { sh.digit = d_hi; sh.above = above; }
    else if (above + c_hi < k_rem && k_rem <= above + c_hi + c_lo) { sh.digit = d_lo; sh.above = above + c_hi; }
    __syncthreads();
    const uint32_t digit = sh.digit;
    prefix = (prefix << dbits) | digit;
    k_rem -= (int)sh.above;
    if (shift == 0) break;
    // Few real elements share the prefix (the usual case after the first pass): rank them against each other
    // directly instead of taking more passes.  Padding slots are the last of the smallest keys and never
    // decide the answer for k <= M, so they stay out.
    const int members = (int)sh.hist[digit] - (digit == 0u && pad_counted && n_pad > 0 ? n_pad : 0);
    if (members <= kRankMax) {                     // workgroup-uniform
      __syncthreads();                             // every thread has read the count
      if (tid == 0) sh.scan_buf[kSelWaves] = 0;
      __syncthreads();
      if constexpr (ITEMS == 0) {
        for (int i0 = 0; i0 < ks.items; i0 += 8) {
          uint32_t kb[8];
          ks.key_batch(i0, kb);
#pragma unroll
          for (int j = 0; j < 8; ++j)
            if (i0 + j < ks.items && ks.page(i0 + j) < ks.M && (kb[j] >> shift) == prefix)
              sh.hist[atomicAdd(&sh.scan_buf[kSelWaves], 1)] = kb[j];
        }
      } else {
#pragma unroll
        for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) {
          const uint32_t v = ks.key(i);
          if (ks.page(i) < ks.M && (v >> shift) == prefix) sh.hist[atomicAdd(&sh.scan_buf[kSelWaves], 1)] = v;
        }
      }
      __syncthreads();
      if (tid < members) {
        const uint32_t v = sh.hist[tid];
        int g = 0, e = 0;
        for (int j = 0; j < members; ++j) { const uint32_t u = sh.hist[j]; g += u > v; e += u == v; }
        if (g < k_rem && k_rem <= g + e) { sh.digit = v; sh.above = (uint32_t)g; }    // equal keys write the same
      }
      __syncthreads();
      vT_out = sh.digit; k_eq_out = k_rem - (int)sh.above;
      return;
    }
  }
  vT_out = prefix; k_eq_out = k_rem;
}

// Writes, in ascending page order, every page whose (rebased) key exceeds vT, plus the first k_eq
// pages (by index) whose key equals vT.  Slots past M are never written.
template <int ITEMS, typename KeyFn>
__device__ __forceinline__ void compact_ordered(const KeySet<ITEMS, KeyFn>& ks, uint32_t vT, int k_eq,
                                                SelectShared& sh, int32_t* __restrict__ out) {
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint64_t lt = (1ull << lane) - 1ull;
  int n_gt = 0, n_eq = 0;
  if constexpr (ITEMS == 0) {
    for (int i0 = 0; i0 < ks.items; i0 += 8) {
      uint32_t kb[8];
      ks.key_batch(i0, kb);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (i0 + j < ks.items) { n_gt += kb[j] > vT; n_eq += kb[j] == vT; }
    }
  } else {
#pragma unroll
    for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) {
      const uint32_t v = ks.key(i);       // per-lane counts (no ballots here: they would all be kept
      n_gt += v > vT;                     // alive for the second loop and exhaust the scalar registers)
      n_eq += v == vT;
    }
  }
  n_gt = wave_sum_i(n_gt);
  n_eq = wave_sum_i(n_eq);
  __syncthreads();
  if (lane == 0) { sh.wave_gt[w] = n_gt; sh.wave_eq[w] = n_eq; }
  __syncthreads();
  int gt_before = 0, eq_before = 0;
  for (int i = 0; i < w; ++i) { gt_before += sh.wave_gt[i]; eq_before += sh.wave_eq[i]; }
  int eq_run = eq_before;
  int o_run = gt_before + min(eq_before, k_eq);
  auto emit = [&](int i, uint32_t v) {
    const bool eq = v == vT;
    const uint64_t m_eq = __ballot(eq);
    const bool take = v > vT || (eq && eq_run + __popcll(m_eq & lt) < k_eq);
    const uint64_t m_take = __ballot(take);
    if (take) out[o_run + __popcll(m_take & lt)] = ks.page(i);
    eq_run += __popcll(m_eq);
    o_run += __popcll(m_take);
  };
  if constexpr (ITEMS == 0) {
    for (int i0 = 0; i0 < ks.items; i0 += 8) {
      uint32_t kb[8];
      ks.key_batch(i0, kb);
#pragma unroll
      for (int j = 0; j < 8; ++j)
        if (i0 + j < ks.items) emit(i0 + j, kb[j]);       // wave-uniform condition
    }
  } else {
#pragma unroll
    for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) {
      emit(i, ks.key(i));
      __builtin_amdgcn_sched_barrier(0);    // keep the iterations in order: hoisting every compare first
    }                                       // needs two scalar register pairs per key
  }
}

}  // namespace ekv
