// Box-threshold selection and refinement (paper App. B.2: a conservative threshold and the page upper
// bounds of Sec. 4.2 Eq. 9 never miss a support page).
//
// Output list of (b,h) = given list  UNION  { p < M_b : a * box[p] > tau_lo[b,h] },  ascending.
// With tau_lo the threshold of a sparse solve over the given list (which never exceeds the full-cache
// threshold), "nothing added" certifies that solve as exact, and otherwise one more solve over the
// output list is exact.
//   mark   (slices of 4096 pages x heads): membership bits of the given list in LDS, threshold test,
//          ordered compaction of the slice into scratch + (total, added) counts;
//   gather (one workgroup per head): prefix over the slices, copy into page_idx_out, flags.
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kBxThreads = 256;
constexpr int kBxItems = 16;
constexpr int kBxSlice = kBxThreads * kBxItems;      // 4096 pages
constexpr int kBxGatherThreads = 1024;
constexpr int kBxMaxSlices = 1024;

static int box_slices(const Dims& dm) { return (dm.Mmax + kBxSlice - 1) / kBxSlice; }

bool select_box_supported(const Dims& dm) { return box_slices(dm) <= kBxMaxSlices; }

size_t select_box_ws_bytes(const Dims& dm) {
  const size_t BH = (size_t)dm.B * dm.Hq, NS = box_slices(dm);
  const size_t b = BH * NS * 2 * sizeof(int32_t) + BH * NS * kBxSlice * sizeof(int32_t);
  return (b + 255) & ~(size_t)255;
}

struct BoxWs {
  int32_t* cnt;    // [BH][NS][2]: pages of the slice in the output, of which newly added
  int32_t* list;   // [BH][NS][kBxSlice]
  int NS;
};

__global__ __launch_bounds__(kBxThreads) void box_mark_kernel(const float* __restrict__ box,
                                                              const int32_t* __restrict__ seq_lens,
                                                              const float* __restrict__ tau_lo,
                                                              const int32_t* __restrict__ page_idx_in,
                                                              const int32_t* __restrict__ n_sel_in, BoxWs ws,
                                                              float a, int Hq, int P, int Mmax, int cap) {
  __shared__ uint32_t bits[kBxSlice / 32];
  __shared__ int wcnt[kBxThreads / 64][2];
  const int bh = blockIdx.y, slice = blockIdx.x, b = bh / Hq, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = seq_lens[b];
  const int M = min((n + P - 1) / P, Mmax);
  int32_t* cnt_out = ws.cnt + ((size_t)bh * ws.NS + slice) * 2;
  const int p_lo = slice * kBxSlice;
  if (p_lo >= M) { if (tid == 0) { cnt_out[0] = 0; cnt_out[1] = 0; } return; }
  const float thr = tau_lo[bh];
  const float* box_r = box + (size_t)bh * Mmax;
  // wavefront w owns 1024 consecutive pages: (load i, lane) order is page order
  const int page0 = p_lo + w * (kBxSlice / (kBxThreads / 64)) + lane;
  float sv[kBxItems];
#pragma unroll
  for (int i = 0; i < kBxItems; ++i) sv[i] = box_r[min(page0 + i * 64, M - 1)];
  if (tid < kBxSlice / 32) bits[tid] = 0u;
  __syncthreads();
  if (page_idx_in != nullptr) {
    const int n_in = min(max(n_sel_in[bh], 0), cap);
    const int32_t* in = page_idx_in + (size_t)bh * cap;
    for (int e = tid; e < n_in; e += kBxThreads) {
      const int p = in[e] - p_lo;
      if (p >= 0 && p < kBxSlice && p + p_lo < M) atomicOr(&bits[p >> 5], 1u << (p & 31));
    }
  }
  __syncthreads();
  uint32_t keep = 0;
  int c_all = 0, c_new = 0;
#pragma unroll
  for (int i = 0; i < kBxItems; ++i) {
    const int p = page0 + i * 64, pl = p - p_lo;
    const bool listed = (bits[pl >> 5] >> (pl & 31)) & 1u;
    const bool above = p < M && a * sv[i] > thr;
    keep |= (uint32_t)(listed || above) << i;
    c_all += listed || above;
    c_new += above && !listed;
  }
  c_all = wave_sum_i(c_all);
  c_new = wave_sum_i(c_new);
  if (lane == 0) { wcnt[w][0] = c_all; wcnt[w][1] = c_new; }
  __syncthreads();
  int o_run = 0, tot = 0, tot_new = 0;
  for (int i = 0; i < kBxThreads / 64; ++i) { if (i < w) o_run += wcnt[i][0]; tot += wcnt[i][0]; tot_new += wcnt[i][1]; }
  int32_t* list = ws.list + ((size_t)bh * ws.NS + slice) * kBxSlice;
  const uint64_t lt = (1ull << lane) - 1ull;
#pragma unroll
  for (int i = 0; i < kBxItems; ++i) {
    const bool in = (keep >> i) & 1u;
    const uint64_t mk = __ballot(in);
    if (in) list[o_run + __popcll(mk & lt)] = page0 + i * 64;
    o_run += __popcll(mk);
  }
  if (tid == 0) { cnt_out[0] = tot; cnt_out[1] = tot_new; }
}

__global__ __launch_bounds__(kBxGatherThreads) void box_gather_kernel(BoxWs ws, int32_t* __restrict__ page_idx_out,
                                                                      int32_t* __restrict__ n_sel_out,
                                                                      int32_t* __restrict__ n_added,
                                                                      int32_t* __restrict__ overflow, int cap) {
  __shared__ int s_off[kBxMaxSlices + 1];
  __shared__ int wsum[kBxGatherThreads / 64][2];
  const int bh = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int NS = ws.NS;
  const int32_t* cnt = ws.cnt + (size_t)bh * NS * 2;
  const int c = tid < NS ? cnt[2 * tid] : 0;
  int cn = tid < NS ? cnt[2 * tid + 1] : 0;
  int inc = c;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(inc, d); if (lane >= d) inc += t; }
  cn = wave_sum_i(cn);
  if (lane == 63) wsum[w][0] = inc;
  if (lane == 0) wsum[w][1] = cn;
  __syncthreads();
  int base = 0, total = 0, added = 0;
  for (int i = 0; i < kBxGatherThreads / 64; ++i) { if (i < w) base += wsum[i][0]; total += wsum[i][0]; added += wsum[i][1]; }
  if (tid < NS) s_off[tid] = base + inc - c;
  if (tid == 0) s_off[NS] = total;
  __syncthreads();
  const int n_out = min(total, cap);
  int32_t* out = page_idx_out + (size_t)bh * cap;
  for (int e = tid; e < n_out; e += kBxGatherThreads) {
    int lo = 0, hi = NS;                       // last slice whose offset is <= e
    while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_off[mid] <= e) lo = mid; else hi = mid; }
    out[e] = ws.list[((size_t)bh * NS + lo) * kBxSlice + (e - s_off[lo])];
  }
  if (tid == 0) { n_sel_out[bh] = n_out; n_added[bh] = added; overflow[bh] = total > cap ? 1 : 0; }
}

void launch_select_box_threshold(const Dims& dm, const float* box, const int32_t* seq_lens, const float* tau_lo,
                                 const int32_t* page_idx_in, const int32_t* n_sel_in, int32_t* page_idx_out,
                                 int32_t* n_sel_out, int32_t* n_added, int32_t* overflow, void* workspace,
                                 hipStream_t st) {
  const int BH = dm.B * dm.Hq;
  BoxWs ws;
  ws.NS = box_slices(dm);
  ws.cnt = (int32_t*)workspace;
  ws.list = ws.cnt + (size_t)BH * ws.NS * 2;
  hipLaunchKernelGGL(box_mark_kernel, dim3(ws.NS, BH), dim3(kBxThreads), 0, st, box, seq_lens, tau_lo, page_idx_in,
                     n_sel_in, ws, dm.a, dm.Hq, dm.P, dm.Mmax, dm.cap);
  hipLaunchKernelGGL(box_gather_kernel, dim3(BH), dim3(kBxGatherThreads), 0, st, ws, page_idx_out, n_sel_out, n_added,
                     overflow, dm.cap);
}

}  // namespace ekv
