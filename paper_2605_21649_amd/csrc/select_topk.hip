// Fixed-budget top-k page selection (paper Sec. 4.3): the k pages of largest box score per
// (sequence, query head), ties towards the lower page index, written in ascending page order.
// One 1024-thread workgroup per (b,h): exact radix selection of the k-th largest score (LDS integer
// histograms), then one ordered compaction pass.  Scores are re-read from L2 in each pass.
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

__global__ __launch_bounds__(kSelThreads) void select_topk_kernel(const float* __restrict__ box,
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
    uint32_t kmin, vT; int k_eq;
    radix_select_kth(keyfn, M, k, sh, kmin, vT, k_eq);
    compact_ordered(keyfn, M, kmin, vT, k_eq, sh, page_idx + (size_t)bh * cap);
  }
  if (threadIdx.x == 0) n_sel[bh] = k;
}

void launch_select_topk(const Dims& dm, const float* box, const int32_t* seq_lens, int k_pages,
                        int32_t* page_idx, int32_t* n_sel, hipStream_t st) {
  hipLaunchKernelGGL(select_topk_kernel, dim3(dm.B * dm.Hq), dim3(kSelThreads), 0, st, box, seq_lens, k_pages,
                     page_idx, n_sel, dm.Hq, dm.P, dm.Mmax, dm.cap);
}

}  // namespace ekv
