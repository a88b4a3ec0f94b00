// Fixed-budget top-k page selection (paper Sec. 4.3): the k pages of largest box score per
// (sequence, query head), ties towards the lower page index, written in ascending page order.
// One 1024-thread workgroup per (b,h): the scores are read once (coalesced) into registers as
// order-preserving keys, the k-th largest is found exactly by radix selection (LDS integer histograms)
// and one ballot-based ordered compaction writes the indices.
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

template <int ITEMS>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void select_topk_kernel(const float* __restrict__ box,
                                                                  const int32_t* __restrict__ seq_lens,
                                                                  int k_pages, int32_t* __restrict__ page_idx,
                                                                  int32_t* __restrict__ n_sel, int Hq, int P,
                                                                  int Mmax, int cap) {
  __shared__ SelectShared sh;
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

void launch_select_topk(const Dims& dm, const float* box, const int32_t* seq_lens, int k_pages,
                        int32_t* page_idx, int32_t* n_sel, hipStream_t st) {
  dim3 grid(dm.B * dm.Hq), block(kSelThreads);
#define EKV_TOPK(ITEMS)                                                                                  \
  hipLaunchKernelGGL(select_topk_kernel<ITEMS>, grid, block, 0, st, box, seq_lens, k_pages, page_idx, n_sel, \
                     dm.Hq, dm.P, dm.Mmax, dm.cap)
  if (dm.Mmax <= 4 * kSelThreads) EKV_TOPK(4);
  else if (dm.Mmax <= 16 * kSelThreads) EKV_TOPK(16);
  else if (dm.Mmax <= 64 * kSelThreads) EKV_TOPK(64);
  else EKV_TOPK(0);
#undef EKV_TOPK
}

}  // namespace ekv
