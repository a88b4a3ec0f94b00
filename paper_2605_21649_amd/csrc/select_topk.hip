// Fixed-budget top-k page selection (paper Sec. 4.3): the k pages of largest box score per
// (sequence, query head), ties towards the lower page index, written in ascending page order.
//
// Small page counts (M <= 16384): one 1024-thread workgroup per (b,h) holds the scores in registers as
// order-preserving keys, finds the k-th largest exactly by radix selection (LDS integer histograms) and
// writes the indices with a ballot-based ordered compaction.
//
// Long contexts: a single compute unit per head is the bottleneck (the paper's "explicit top-k
// bottleneck"), so the work is split over slices of 4096 pages and three launches:
//   hist     (slices x heads workgroups)  2048-bin histogram of each slice over a key range estimated from
//                                         the first 1024 pages (keys outside are clamped into the edge bins,
//                                         which keeps the binning monotone), stored as counts-above per bin;
//   find     (one workgroup per head)     bin of the k-th largest from the summed counts, its members are
//                                         gathered and ranked exactly -> the k-th key, the tie quota and the
//                                         output offset of every slice;
//   compact  (slices x heads workgroups)  ordered compaction of each slice against that key.
// If the bin of the k-th key holds more members than the ranking list (massive ties), the find workgroup
// does that head by the single-workgroup algorithm itself and the compaction launch skips it.
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

// ------------------------------------------------------------------------------------------
// single-workgroup algorithm
// ------------------------------------------------------------------------------------------
template <int ITEMS>
__device__ __forceinline__ void topk_single(const float* __restrict__ box, const int32_t* __restrict__ seq_lens,
                                            int k_pages, int32_t* __restrict__ page_idx,
                                            int32_t* __restrict__ n_sel, int Hq, int P, int Mmax, int cap,
                                            SelectShared& sh) {
  const int bh = blockIdx.x, b = bh / Hq;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const int k = min(min(k_pages, M), cap);
  const float* s = box + (size_t)bh * Mmax;
  auto keyfn = [s](int p) { return float_to_key(s[p]); };
  if (k > 0) {
    KeySet<ITEMS, decltype(keyfn)> ks(keyfn, M);
    uint32_t vT; int k_eq;
    radix_select_kth(ks, k, sh, vT, k_eq);
    compact_ordered(ks, vT, k_eq, sh, page_idx + (size_t)bh * cap);
  }
  if (threadIdx.x == 0) n_sel[bh] = k;
}

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void select_topk_kernel(
    const float* __restrict__ box, const int32_t* __restrict__ seq_lens, int k_pages,
    int32_t* __restrict__ page_idx, int32_t* __restrict__ n_sel, int Hq, int P, int Mmax, int cap) {
  __shared__ SelectShared sh;
  topk_single<ITEMS>(box, seq_lens, k_pages, page_idx, n_sel, Hq, P, Mmax, cap, sh);
}

// ------------------------------------------------------------------------------------------
// short rows: one wavefront per (b,h)
// ------------------------------------------------------------------------------------------
// Rows of at most 64*KPL pages: the keys of a row sit in the registers of ONE wavefront (lane l holds pages
// i*64 + l), the k-th largest key is found bit by bit from the top (the largest v with #{key >= v} >= k; a
// ballot and a population count per register and bit), and ballots give the ordered output.  No LDS, no
// barrier, four rows per 256-thread workgroup: with hundreds or thousands of short rows (many sequences of a
// few thousand tokens) the 1024-thread workgroup per row of the kernel above fills the GPU several times over.
template <int KPL>
__global__ __launch_bounds__(256) void select_topk_wave_kernel(const float* __restrict__ box,
                                                               const int32_t* __restrict__ seq_lens, int k_pages,
                                                               int32_t* __restrict__ page_idx,
                                                               int32_t* __restrict__ n_sel, int Hq, int P, int Mmax,
                                                               int cap, int BH) {
  const int lane = threadIdx.x & 63;
  const int bh = blockIdx.x * 4 + (int)(threadIdx.x >> 6);
  if (bh >= BH) return;                                   // wave-uniform
  const int n = seq_lens[bh / Hq];
  const int M = min((n + P - 1) / P, Mmax);
  const int k = min(min(k_pages, M), cap);
  if (k <= 0) { if (lane == 0) n_sel[bh] = 0; return; }
  const float* s = box + (size_t)bh * Mmax;
  const uint64_t lt = (1ull << lane) - 1ull;
  float raw[KPL];
#pragma unroll
  for (int i = 0; i < KPL; ++i) raw[i] = s[min(i * 64 + lane, M - 1)];
  uint32_t key[KPL];                                      // slots past M: 0, below every real key
#pragma unroll
  for (int i = 0; i < KPL; ++i) key[i] = i * 64 + lane < M ? float_to_key(raw[i]) : 0u;
  uint32_t kth = 0u;
  bool exact = false;                                     // exactly k keys are >= kth: the set is decided
  for (int bit = 31; bit >= 0 && !exact; --bit) {
    const uint32_t cand = kth | (1u << bit);
    int cnt = 0;
#pragma unroll
    for (int i = 0; i < KPL; ++i) cnt += __popcll(__ballot(key[i] >= cand));
    if (cnt >= k) { kth = cand; exact = cnt == k; }       // wave-uniform
  }
  if (exact) kth -= 1u;                                   // the k keys above kth - 1 (kth >= 1 here)
  int n_gt = 0;
#pragma unroll
  for (int i = 0; i < KPL; ++i) n_gt += __popcll(__ballot(key[i] > kth));
  const int k_eq = k - n_gt;                              // pages equal to the k-th key that are taken: lowest indices
  int32_t* out = page_idx + (size_t)bh * cap;
  int o_run = 0, eq_run = 0;
#pragma unroll
  for (int i = 0; i < KPL; ++i) {
    const bool valid = i * 64 + lane < M;
    const bool eq = valid && key[i] == kth;
    const uint64_t m_eq = __ballot(eq);
    const bool take = (valid && key[i] > kth) || (eq && eq_run + __popcll(m_eq & lt) < k_eq);
    const uint64_t m_take = __ballot(take);
    if (take) out[o_run + __popcll(m_take & lt)] = i * 64 + lane;
    eq_run += __popcll(m_eq);
    o_run += __popcll(m_take);
  }
  if (lane == 0) n_sel[bh] = k;
}

// ------------------------------------------------------------------------------------------
// sliced kernels
// ------------------------------------------------------------------------------------------
constexpr int kTkThreads = 256;
constexpr int kTkWaves = kTkThreads / 64;
constexpr int kTkItems = 16;                                  // keys per lane
constexpr int kTkSlice = kTkThreads * kTkItems;               // pages per slice: 4096
constexpr int kTkSample = 1024;                               // pages the key range is estimated from (16 runs of 64)
constexpr int kTkMembers = 1024;                              // ranking list of the find kernel
constexpr int kTkMaxSlices = 64;
constexpr int kTkPrefix = 512;                                // best pages of a slice kept sorted by bin

struct TopkHead {             // per (b,h) state passed between the launches
  uint32_t lo;                // bin(key) = key <= lo ? 0 : min(kBins-1, (key - lo) >> shift)
  int32_t shift;
  uint32_t key_t;             // the k-th largest key
  int32_t k_eq;               // how many pages with key == key_t are taken (lowest indices first)
  int32_t redo;               // 1: the single-workgroup algorithm must redo this head
  int32_t pad[3];
};
struct TopkWs {
  TopkHead* head;             // [BH]
  uint16_t* above;            // [BH][S][kBins]   pages of the slice in bins above this one (<= 4096)
  int32_t* slice_off;         // [BH][S]          output offset of the slice
  int32_t* slice_eq;          // [BH][S]          pages with key == key_t in earlier slices
  uint32_t* prefix_key;       // [BH][S][kTkPrefix]  the slice's pages of the highest bins, grouped by bin
  int32_t* prefix_page;       //                     (descending; arbitrary order inside a bin)
  int S;
};

__device__ __forceinline__ int topk_bin(uint32_t key, uint32_t lo, int shift) {
  return key <= lo ? 0 : (int)min((uint32_t)(kBins - 1), (key - lo) >> shift);
}

// The 16 keys of this lane: wavefront w of slice s owns pages s*4096 + w*1024 + i*64 + lane (ascending in
// (w, i, lane) order).  Unconditional clamped loads; slots past M are flagged invalid.
__device__ __forceinline__ void load_slice_keys(const float* __restrict__ s, int M, int page0,
                                                uint32_t (&key)[kTkItems], uint32_t& valid_mask) {
  float raw[kTkItems];
#pragma unroll
  for (int i = 0; i < kTkItems; ++i) raw[i] = s[min(page0 + i * 64, M - 1)];
  valid_mask = 0;
#pragma unroll
  for (int i = 0; i < kTkItems; ++i) {
    key[i] = float_to_key(raw[i]);
    if (page0 + i * 64 < M) valid_mask |= 1u << i;
  }
}

__global__ __launch_bounds__(kTkThreads) void topk_hist_kernel(const float* __restrict__ box,
                                                               const int32_t* __restrict__ seq_lens, TopkWs ws,
                                                               int Hq, int P, int Mmax) {
  __shared__ uint32_t hist[kBins];
  __shared__ uint32_t pre_key[kTkPrefix];
  __shared__ int32_t pre_page[kTkPrefix];
  __shared__ uint32_t red[2][kTkWaves];
  __shared__ int wsum[kTkWaves];
  const int bh = blockIdx.y, slice = blockIdx.x, b = bh / Hq, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const float* s = box + (size_t)bh * Mmax;
  if (slice * kTkSlice >= M) {            // empty slice: all counts are zero
    for (int i = tid; i < kBins; i += kTkThreads) ws.above[((size_t)bh * ws.S + slice) * kBins + i] = (uint16_t)0;
    return;
  }
  // key range of kTkSample pages -- 16 runs of 64 consecutive pages spread evenly over the sequence, so that a
  // trend along the sequence (recent pages scoring higher, a block of high pages at the start) is inside the
  // range -- widened by half its width on both sides
  uint32_t lo = 0xffffffffu, hi = 0u;
  {
    const int run_stride = max(64, (M / (kTkSample / 64)) & ~63);
    float sv[kTkSample / kTkThreads];
#pragma unroll
    for (int i = 0; i < kTkSample / kTkThreads; ++i) {
      const int j = tid + i * kTkThreads;
      sv[i] = s[min((j >> 6) * run_stride + (j & 63), M - 1)];
    }
#pragma unroll
    for (int i = 0; i < kTkSample / kTkThreads; ++i) {
      const uint32_t kk = float_to_key(sv[i]);
      lo = min(lo, kk); hi = max(hi, kk);
    }
  }
  for (int d = 32; d >= 1; d >>= 1) {
    lo = min(lo, (uint32_t)__shfl_xor((int)lo, d));
    hi = max(hi, (uint32_t)__shfl_xor((int)hi, d));
  }
  if (lane == 0) { red[0][w] = lo; red[1][w] = hi; }
  for (int i = tid; i < kBins; i += kTkThreads) hist[i] = 0;
  __syncthreads();
  for (int i = 0; i < kTkWaves; ++i) { lo = min(lo, red[0][i]); hi = max(hi, red[1][i]); }
  const uint32_t half = (hi - lo) >> 1;
  const uint32_t lo_w = lo > half ? lo - half : 0u;
  const uint32_t hi_w = hi + half >= hi ? hi + half : 0xffffffffu;
  const uint32_t range = hi_w - lo_w;
  const int bits = range ? 32 - __clz(range) : 0;
  const int shift = max(bits - kDigitBits, 0);
  if (slice == 0 && tid == 0) { ws.head[bh].lo = lo_w; ws.head[bh].shift = shift; ws.head[bh].redo = 0; }

  uint32_t key[kTkItems], vmask;
  load_slice_keys(s, M, slice * kTkSlice + w * (kTkSlice / kTkWaves) + lane, key, vmask);
#pragma unroll
  for (int i = 0; i < kTkItems; ++i)
    if (vmask & (1u << i)) atomicAdd(&hist[topk_bin(key[i], lo_w, shift)], 1u);
  __syncthreads();
  // counts above each bin: thread t owns the 8 bins [8t, 8t+8); suffix sums over the block
  constexpr int BPT = kBins / kTkThreads;
  uint32_t c[BPT];
  int tot = 0;
#pragma unroll
  for (int i = 0; i < BPT; ++i) { c[i] = hist[tid * BPT + i]; tot += (int)c[i]; }
  int inc = tot;                                   // inclusive sum over this and all HIGHER lanes
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_down(inc, d); if (lane + d < 64) inc += t; }
  if (lane == 0) wsum[w] = inc;
  __syncthreads();
  int higher = 0;                                  // pages in bins owned by higher wavefronts
  for (int i = w + 1; i < kTkWaves; ++i) higher += wsum[i];
  uint32_t run = (uint32_t)(higher + inc - tot);   // pages in bins above this thread's highest bin
  uint32_t ab[BPT];
#pragma unroll
  for (int i = BPT - 1; i >= 0; --i) { ab[i] = run; run += c[i]; }
  static_assert(BPT == 8, "one 16-byte store of eight 16-bit counts per thread");
  uint16_t* out = ws.above + ((size_t)bh * ws.S + slice) * kBins + tid * BPT;
  *reinterpret_cast<uint4*>(out) = make_uint4(ab[0] | (ab[1] << 16), ab[2] | (ab[3] << 16), ab[4] | (ab[5] << 16),
                                              ab[6] | (ab[7] << 16));
  // The kTkPrefix best pages of the slice, grouped by bin in descending bin order: a page of bin g goes to
  // position above[g] + (arrival number inside the bin).  The find kernel then reads the members of the
  // bin of the k-th key from these lists instead of scanning every score again.
  __syncthreads();                                   // all reads of the counts are done
#pragma unroll
  for (int i = 0; i < BPT; ++i) hist[tid * BPT + i] = ab[i];
  __syncthreads();
  const int page0 = slice * kTkSlice + w * (kTkSlice / kTkWaves) + lane;
#pragma unroll
  for (int i = 0; i < kTkItems; ++i) {
    if (vmask & (1u << i)) {
      const uint32_t pos = atomicAdd(&hist[topk_bin(key[i], lo_w, shift)], 1u);
      if (pos < (uint32_t)kTkPrefix) { pre_key[pos] = key[i]; pre_page[pos] = page0 + i * 64; }
    }
  }
  __syncthreads();
  const int n_valid = min(kTkSlice, M - slice * kTkSlice);
  uint32_t* pk = ws.prefix_key + ((size_t)bh * ws.S + slice) * kTkPrefix;
  int32_t* pp = ws.prefix_page + ((size_t)bh * ws.S + slice) * kTkPrefix;
  for (int t = tid; t < min(kTkPrefix, n_valid); t += kTkThreads) { pk[t] = pre_key[t]; pp[t] = pre_page[t]; }
}

__global__ __launch_bounds__(kSelThreads) void topk_find_kernel(const float* __restrict__ box,
                                                                const int32_t* __restrict__ seq_lens, int k_pages,
                                                                TopkWs ws, int32_t* __restrict__ page_idx,
                                                                int32_t* __restrict__ n_sel, int Hq, int P, int Mmax,
                                                                int cap) {
  __shared__ uint32_t tot_above[kBins];                // summed over the slices
  __shared__ uint32_t mem_key[kTkMembers];
  __shared__ int32_t mem_page[kTkMembers];
  __shared__ int s_gt[kTkMaxSlices], s_eq[kTkMaxSlices];
  __shared__ int s_bin, s_cnt, s_m;
  __shared__ uint32_t s_keyt;
  const int bh = blockIdx.x, b = bh / Hq, tid = threadIdx.x;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const int k = min(min(k_pages, M), cap);
  const int S = ws.S;
  const float* s = box + (size_t)bh * Mmax;
  if (M <= 0) { if (tid == 0) n_sel[bh] = 0; return; }
  const TopkHead hd = ws.head[bh];

  // counts above each bin, summed over the slices (thread t owns bins 2t and 2t+1)
  uint32_t a0 = 0, a1 = 0;
  {
    const uint16_t* ab = ws.above + (size_t)bh * S * kBins + 2 * tid;
    for (int s0 = 0; s0 < S; s0 += 16) {
      uint32_t v[16];                                       // two 16-bit counts per load
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = *reinterpret_cast<const uint32_t*>(ab + (size_t)min(s0 + i, S - 1) * kBins);
#pragma unroll
      for (int i = 0; i < 16; ++i) if (s0 + i < S) { a0 += v[i] & 0xffffu; a1 += v[i] >> 16; }
    }
  }
  tot_above[2 * tid] = a0; tot_above[2 * tid + 1] = a1;
  if (tid == 0) { s_m = 0; s_bin = 0; s_cnt = 0; s_keyt = 0u; }
  if (tid < kTkMaxSlices) { s_gt[tid] = 0; s_eq[tid] = 0; }
  __syncthreads();
  // bin b1 of the k-th largest: above[b1] < k <= above[b1 - 1]   (above[-1] := M)
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int bin = 2 * tid + i;
    const uint32_t ab = tot_above[bin];
    const uint32_t below = bin == 0 ? (uint32_t)M : tot_above[bin - 1];
    if (ab < (uint32_t)k && (uint32_t)k <= below) { s_bin = bin; s_cnt = (int)(below - ab); }
  }
  __syncthreads();
  const int b1 = s_bin;
  int m = s_cnt;
  const int k_bin = k - (int)tot_above[b1];            // rank of the answer inside bin b1 (1-based)
  int k_rem = k_bin;                                   // ... inside the list of members that is ranked below
  // Members of bin b1.  In slice s they sit at positions [above_s[b1], above_s[b1 - 1]) of its prefix list
  // (above_s[-1] := pages of the slice): copied from there when the range ends inside the list.  A slice
  // whose range does not (more than kTkPrefix of its pages at or above the bin: the top pages crowd into a
  // few slices, or the budget is very large) has its 4096 scores scanned instead.
  __shared__ int s_lo[kTkMaxSlices], s_cnt_s[kTkMaxSlices], s_start[kTkMaxSlices + 1], s_all[kTkMaxSlices];
  __shared__ unsigned long long s_scan_mask;             // slices to scan (kTkMaxSlices <= 64: the first wavefront's ballot)
  static_assert(kTkMaxSlices <= 64, "one ballot covers the slices");
  if (tid < 64) {
    bool scan = false;
    if (tid < S) {
      const uint16_t* ab = ws.above + ((size_t)bh * S + tid) * kBins;
      const int lo_s = (int)ab[b1];
      const int valid_s = max(0, min(kTkSlice, M - tid * kTkSlice));
      const int hi_s = b1 == 0 ? valid_s : (int)ab[b1 - 1];
      scan = hi_s > kTkPrefix && hi_s > lo_s;
      s_lo[tid] = lo_s; s_cnt_s[tid] = scan ? 0 : hi_s - lo_s; s_all[tid] = max(hi_s - lo_s, 0);
    }
    const unsigned long long mask = __ballot(scan);
    if (tid == 0) s_scan_mask = mask;
    // exclusive prefix of the copied counts (one lane per slice: a serial loop over LDS costs a latency per slice)
    const int cs = tid < S ? s_cnt_s[tid] : 0;
    int inc = cs;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(inc, d); if (tid >= d) inc += t; }
    if (tid < S) s_start[tid] = inc - cs;
    const int run = __shfl(inc, 63);
    if (tid == 0) { s_start[S] = run; s_m = run; }       // the scanned slices append behind the copied ones
  }
  __syncthreads();
  // Every member of bin b1, wherever it is kept: fn(has, key, page, slice) is called by whole wavefronts (`has` says
  // whether this lane holds a member); a wavefront is inside one slice at a time.
  auto for_each_member = [&](auto&& fn) {
    for (int sl = tid >> 6; sl < S; sl += kSelWaves) {
      const uint32_t* pk = ws.prefix_key + ((size_t)bh * S + sl) * kTkPrefix + s_lo[sl];
      const int32_t* pp = ws.prefix_page + ((size_t)bh * S + sl) * kTkPrefix + s_lo[sl];
      const int cnt = s_cnt_s[sl];
      for (int e0 = 0; e0 < cnt; e0 += 64) {
        const int e = e0 + (tid & 63);
        const bool has = e < cnt;
        fn(has, has ? pk[e] : 0u, has ? pp[e] : 0, sl);
      }
    }
    for (unsigned long long todo = s_scan_mask; todo != 0; todo &= todo - 1) {     // workgroup-uniform, usually empty
      const int sl = __builtin_ctzll(todo);
      constexpr int PER = kTkSlice / kSelThreads;        // 4 scores per thread
      float raw[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) raw[i] = s[min(sl * kTkSlice + tid + i * kSelThreads, M - 1)];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int p = sl * kTkSlice + tid + i * kSelThreads;
        const uint32_t kk = float_to_key(raw[i]);
        fn(p < M && topk_bin(kk, hd.lo, hd.shift) == b1, kk, p, sl);
      }
    }
  };
  bool all_equal = false;
  if (m <= kTkMembers) {
    // the usual case: the members fit the ranking list (arrival order is irrelevant: the ranks below are exact)
    for (int sl = tid >> 6; sl < S; sl += kSelWaves) {
      const uint32_t* pk = ws.prefix_key + ((size_t)bh * S + sl) * kTkPrefix + s_lo[sl];
      const int32_t* pp = ws.prefix_page + ((size_t)bh * S + sl) * kTkPrefix + s_lo[sl];
      for (int e = tid & 63; e < s_cnt_s[sl]; e += 64) {
        const int slot = s_start[sl] + e;
        if (slot < kTkMembers) { mem_key[slot] = pk[e]; mem_page[slot] = pp[e]; }
      }
    }
    for (unsigned long long todo = s_scan_mask; todo != 0; todo &= todo - 1) {     // workgroup-uniform, usually empty
      const int sl = __builtin_ctzll(todo);
      constexpr int PER = kTkSlice / kSelThreads;        // 4 scores per thread
      float raw[PER];
#pragma unroll
      for (int i = 0; i < PER; ++i) raw[i] = s[min(sl * kTkSlice + tid + i * kSelThreads, M - 1)];
#pragma unroll
      for (int i = 0; i < PER; ++i) {
        const int p = sl * kTkSlice + tid + i * kSelThreads;
        const uint32_t kk = float_to_key(raw[i]);
        if (p < M && topk_bin(kk, hd.lo, hd.shift) == b1) {
          const int slot = atomicAdd(&s_m, 1);
          if (slot < kTkMembers) { mem_key[slot] = kk; mem_page[slot] = p; }
        }
      }
    }
  } else {
    // More members than the ranking list holds: many scores that are equal or nearly so.  The members are streamed
    // (not stored) once for their smallest and largest key and a histogram of the bits below the bin's: if all keys
    // are equal that key is the answer and the per-slice counts are already known; otherwise the sub-bin of the
    // k-th key usually holds few enough members to rank, collected by a second pass that also counts, per slice,
    // the members of the higher sub-bins.  Only a sub-bin that is still too large sends the head to the
    // single-workgroup algorithm (which the compaction launch then skips).
    __shared__ uint32_t s_kmin, s_kmax;
    __shared__ int s_sub, s_above2, wsum2[kSelWaves];
    const bool edge = b1 == 0 || b1 == kBins - 1;        // clamped bins: keys outside the sampled range, no sub-bins
    const int sub_shift = max(hd.shift - kDigitBits, 0);
    const uint32_t sub_mask = hd.shift >= kDigitBits ? (uint32_t)(kBins - 1) : ((1u << hd.shift) - 1u);
    auto sub_of = [&](uint32_t kk) { return (int)(((kk - hd.lo) >> sub_shift) & sub_mask); };
    tot_above[2 * tid] = 0; tot_above[2 * tid + 1] = 0;  // reused as the sub-bin histogram
    if (tid == 0) { s_kmin = 0xffffffffu; s_kmax = 0u; s_sub = -1; s_above2 = 0; }
    __syncthreads();
    for_each_member([&](bool has, uint32_t kk, int, int) {
      uint32_t lo_k = has ? kk : 0xffffffffu, hi_k = has ? kk : 0u;
      for (int d = 32; d >= 1; d >>= 1) {
        lo_k = min(lo_k, (uint32_t)__shfl_xor((int)lo_k, d));
        hi_k = max(hi_k, (uint32_t)__shfl_xor((int)hi_k, d));
      }
      if ((tid & 63) == 0 && lo_k <= hi_k) { atomicMin(&s_kmin, lo_k); atomicMax(&s_kmax, hi_k); }
      if (has && !edge) atomicAdd(&tot_above[sub_of(kk)], 1u);
    });
    __syncthreads();
    all_equal = s_kmin == s_kmax;
    if (all_equal) {
      if (tid == 0) s_keyt = s_kmin;
      if (tid < S) { s_gt[tid] = 0; s_eq[tid] = s_all[tid]; }
    } else {
      // sub-bin of the k_rem-th largest member: thread t owns sub-bins 2t and 2t+1; counts above by a suffix scan
      int sub = -1, above2 = 0, m2 = m;
      if (!edge) {
        const uint32_t c0 = tot_above[2 * tid], c1 = tot_above[2 * tid + 1];
        int inc = (int)(c0 + c1);
        const int tot = inc;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_down(inc, d); if ((tid & 63) + d < 64) inc += t; }
        if ((tid & 63) == 0) wsum2[tid >> 6] = inc;
        __syncthreads();
        int higher = 0;
        for (int i = (tid >> 6) + 1; i < kSelWaves; ++i) higher += wsum2[i];
        const int ab1 = higher + inc - tot;              // members in sub-bins above 2t+1
        const int ab0 = ab1 + (int)c1;                   // ... above 2t
        if (ab1 < k_rem && k_rem <= ab1 + (int)c1) { s_sub = 2 * tid + 1; s_above2 = ab1; s_cnt = (int)c1; }
        if (ab0 < k_rem && k_rem <= ab0 + (int)c0) { s_sub = 2 * tid; s_above2 = ab0; s_cnt = (int)c0; }
        __syncthreads();
        sub = s_sub; above2 = s_above2; m2 = s_cnt;
      }
      // second pass: per slice, the members of the higher sub-bins; the members of the k-th key's sub-bin are
      // collected for ranking if they fit -- if they do not, they may still all be one value (then their per-slice
      // counts are all that is needed)
      const bool collect = sub >= 0 && m2 <= kTkMembers;
      if (tid == 0) { s_m = 0; s_kmin = 0xffffffffu; s_kmax = 0u; }
      __syncthreads();
      if (sub >= 0) {
        for_each_member([&](bool has, uint32_t kk, int page, int sl) {
          const int sb = has ? sub_of(kk) : -1;
          const unsigned long long up = __ballot(has && sb > sub);
          if ((tid & 63) == 0 && up) atomicAdd(&s_gt[sl], __popcll(up));     // a wavefront is inside one slice
          const bool mine = has && sb == sub;
          if (collect) {
            if (mine) {
              const int slot = atomicAdd(&s_m, 1);
              if (slot < kTkMembers) { mem_key[slot] = kk; mem_page[slot] = page; }
            }
          } else {
            uint32_t lo_k = mine ? kk : 0xffffffffu, hi_k = mine ? kk : 0u;
            for (int d = 32; d >= 1; d >>= 1) {
              lo_k = min(lo_k, (uint32_t)__shfl_xor((int)lo_k, d));
              hi_k = max(hi_k, (uint32_t)__shfl_xor((int)hi_k, d));
            }
            const unsigned long long eqm = __ballot(mine);
            if ((tid & 63) == 0 && eqm) { atomicMin(&s_kmin, lo_k); atomicMax(&s_kmax, hi_k); atomicAdd(&s_eq[sl], __popcll(eqm)); }
          }
        });
        __syncthreads();
      }
      if (collect) {
        m = m2; k_rem -= above2;
      } else if (sub >= 0 && s_kmin == s_kmax) {
        all_equal = true;                                  // one value fills the sub-bin: it is the k-th key
        if (tid == 0) s_keyt = s_kmin;
      } else {
        if (tid == 0) ws.head[bh].redo = 1;
        __shared__ SelectShared sh;
        topk_single<0>(box, seq_lens, k_pages, page_idx, n_sel, Hq, P, Mmax, cap, sh);
        return;
      }
    }
  }
  __syncthreads();
  // exact rank of every member: larger key first, lower page first among equal keys
  // (16 lanes share a member and split the others among them; 64 members per sweep of the workgroup)
  for (int i0 = 0; i0 < (all_equal ? 0 : m); i0 += kSelThreads / 16) {
    const int i = min(i0 + (tid >> 4), m - 1), l = tid & 15;
    const uint32_t kk = mem_key[i]; const int pp = mem_page[i];
    int rank = 0;
    for (int j0 = 0; j0 < m; j0 += 64) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int jj = j0 + u * 16 + l, jc = min(jj, m - 1);
        const uint32_t kj = mem_key[jc]; const int pj = mem_page[jc];
        rank += jj < m && ((kj > kk) || (kj == kk && pj < pp));
      }
    }
    rank += dpp_move_i<0xB1>(rank);
    rank += dpp_move_i<0x4E>(rank);
    rank += dpp_move_i<0x141>(rank);
    rank += dpp_move_i<0x140>(rank);
    if (l == 0 && i0 + (tid >> 4) < m && rank == k_rem - 1) s_keyt = kk;   // the k-th largest key overall
  }
  __syncthreads();
  const uint32_t key_t = s_keyt;
  if (!all_equal && tid < m) {
    const uint32_t kk = mem_key[tid];
    const int sl = mem_page[tid] / kTkSlice;
    if (kk > key_t) atomicAdd(&s_gt[sl], 1);
    else if (kk == key_t) atomicAdd(&s_eq[sl], 1);
  }
  __syncthreads();
  // per-slice output offsets: the global loads are done in parallel, the short serial prefix runs on LDS
  if (tid < 64) {                                      // one lane per slice, wave scans instead of serial loops
    const int ab_s = tid < S ? (int)ws.above[((size_t)bh * S + tid) * kBins + b1] : 0;
    const int gt_s = tid < S ? s_gt[tid] : 0, eq_s = tid < S ? s_eq[tid] : 0;
    int gt_inc = gt_s, eq_inc = eq_s;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int tg = __shfl_up(gt_inc, d), te = __shfl_up(eq_inc, d);
      if (tid >= d) { gt_inc += tg; eq_inc += te; }
    }
    const int k_eq = k_bin - __shfl(gt_inc, 63);       // pages equal to key_t that are taken
    const int eq_before = eq_inc - eq_s;
    const int take_eq = max(0, min(eq_s, k_eq - eq_before));
    int off_inc = ab_s + gt_s + take_eq;
    const int mine = off_inc;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(off_inc, d); if (tid >= d) off_inc += t; }
    if (tid < S) {
      ws.slice_off[(size_t)bh * S + tid] = off_inc - mine;
      ws.slice_eq[(size_t)bh * S + tid] = eq_before;
    }
    if (tid == 0) { ws.head[bh].key_t = key_t; ws.head[bh].k_eq = k_eq; n_sel[bh] = k; }
  }
}

__global__ __launch_bounds__(kTkThreads) void topk_compact_kernel(const float* __restrict__ box,
                                                                  const int32_t* __restrict__ seq_lens, TopkWs ws,
                                                                  int32_t* __restrict__ page_idx, int Hq, int P,
                                                                  int Mmax, int cap) {
  __shared__ int w_take[kTkWaves], w_eq[kTkWaves];
  const int bh = blockIdx.y, slice = blockIdx.x, b = bh / Hq, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  if (slice * kTkSlice >= M) return;
  const TopkHead hd = ws.head[bh];
  if (hd.redo) return;
  const float* s = box + (size_t)bh * Mmax;
  const int page0 = slice * kTkSlice + w * (kTkSlice / kTkWaves) + lane;
  uint32_t key[kTkItems], vmask;
  load_slice_keys(s, M, page0, key, vmask);
  const uint64_t lt = (1ull << lane) - 1ull;
  // per-wavefront totals of (key > key_t) and (key == key_t)
  int n_gt = 0, n_eq = 0;
#pragma unroll
  for (int i = 0; i < kTkItems; ++i) {
    const bool ok = vmask & (1u << i);
    n_gt += ok && key[i] > hd.key_t;
    n_eq += ok && key[i] == hd.key_t;
  }
  n_gt = wave_sum_i(n_gt); n_eq = wave_sum_i(n_eq);
  if (lane == 0) { w_take[w] = n_gt; w_eq[w] = n_eq; }
  __syncthreads();
  int eq_run = ws.slice_eq[(size_t)bh * ws.S + slice];
  int o_run = ws.slice_off[(size_t)bh * ws.S + slice];
  for (int i = 0; i < w; ++i) {
    const int take_eq = max(0, min(w_eq[i], hd.k_eq - eq_run));
    o_run += w_take[i] + take_eq;
    eq_run += w_eq[i];
  }
  int32_t* out = page_idx + (size_t)bh * cap;
#pragma unroll
  for (int i = 0; i < kTkItems; ++i) {
    const bool ok = vmask & (1u << i);
    const bool eq = ok && key[i] == hd.key_t;
    const uint64_t m_eq = __ballot(eq);
    const bool take = (ok && key[i] > hd.key_t) || (eq && eq_run + __popcll(m_eq & lt) < hd.k_eq);
    const uint64_t m_take = __ballot(take);
    if (take) out[o_run + __popcll(m_take & lt)] = page0 + i * 64;
    eq_run += __popcll(m_eq);
    o_run += __popcll(m_take);
  }
}

static int topk_slices(const Dims& dm) { return (dm.Mmax + kTkSlice - 1) / kTkSlice; }
static bool topk_sliced(const Dims& dm) { return dm.Mmax > 16 * kSelThreads && topk_slices(dm) <= kTkMaxSlices; }

size_t select_topk_ws_bytes(const Dims& dm) {
  if (!topk_sliced(dm)) return 256;
  const size_t BH = (size_t)dm.B * dm.Hq, S = topk_slices(dm);
  size_t b = BH * sizeof(TopkHead) + BH * S * kBins * sizeof(uint16_t) + 2 * BH * S * sizeof(int32_t) +
             2 * BH * S * kTkPrefix * sizeof(int32_t);
  return (b + 255) & ~(size_t)255;
}

void launch_select_topk(const Dims& dm, const float* box, const int32_t* seq_lens, int k_pages,
                        int32_t* page_idx, int32_t* n_sel, void* workspace, hipStream_t st) {
  dim3 grid(dm.B * dm.Hq), block(kSelThreads);
#define EKV_TOPK(ITEMS)                                                                                        \
  hipLaunchKernelGGL(select_topk_kernel<ITEMS>, grid, block, 0, st, box, seq_lens, k_pages, page_idx, n_sel, dm.Hq, \
                     dm.P, dm.Mmax, dm.cap)
  const int n_rows = dm.B * dm.Hq;
#define EKV_TOPK_WAVE(KPL)                                                                                          \
  hipLaunchKernelGGL(select_topk_wave_kernel<KPL>, dim3((n_rows + 3) / 4), dim3(256), 0, st, box, seq_lens, k_pages, \
                     page_idx, n_sel, dm.Hq, dm.P, dm.Mmax, dm.cap, n_rows)
  if (n_rows > 512) {              // up to 512 rows the workgroup kernel below takes one round and is as fast
    if (dm.Mmax <= 256) { EKV_TOPK_WAVE(4); return; }
    if (dm.Mmax <= 512) { EKV_TOPK_WAVE(8); return; }
    if (dm.Mmax <= 1024) { EKV_TOPK_WAVE(16); return; }
    if (dm.Mmax <= 2048) { EKV_TOPK_WAVE(32); return; }
  }
#undef EKV_TOPK_WAVE
  if (!topk_sliced(dm)) {
    if (dm.Mmax <= 2 * kSelThreads) EKV_TOPK(2);
    else if (dm.Mmax <= 4 * kSelThreads) EKV_TOPK(4);
    else if (dm.Mmax <= 8 * kSelThreads) EKV_TOPK(8);
    else if (dm.Mmax <= 16 * kSelThreads) EKV_TOPK(16);
    else EKV_TOPK(0);
    return;
  }
#undef EKV_TOPK
  const size_t BH = (size_t)dm.B * dm.Hq;
  TopkWs ws;
  ws.S = topk_slices(dm);
  ws.head = (TopkHead*)workspace;
  ws.above = (uint16_t*)(ws.head + BH);
  ws.slice_off = (int32_t*)(ws.above + BH * ws.S * kBins);
  ws.slice_eq = ws.slice_off + BH * ws.S;
  ws.prefix_key = (uint32_t*)(ws.slice_eq + BH * ws.S);
  ws.prefix_page = (int32_t*)(ws.prefix_key + BH * ws.S * kTkPrefix);
  dim3 sgrid(ws.S, dm.B * dm.Hq), sblock(kTkThreads);
  hipLaunchKernelGGL(topk_hist_kernel, sgrid, sblock, 0, st, box, seq_lens, ws, dm.Hq, dm.P, dm.Mmax);
  hipLaunchKernelGGL(topk_find_kernel, grid, block, 0, st, box, seq_lens, k_pages, ws, page_idx, n_sel, dm.Hq, dm.P,
                     dm.Mmax, dm.cap);
  hipLaunchKernelGGL(topk_compact_kernel, sgrid, sblock, 0, st, box, seq_lens, ws, page_idx, dm.Hq, dm.P, dm.Mmax,
                     dm.cap);
}

}  // namespace ekv
