// Softmax attention restricted to the selected pages: the sparse softmax baseline the paper compares
// entmax selection against (Sec. 5.5, App. E.1) and whose kept mass enters Eq. 8.
// Split over chunks of pages with the usual running-maximum rescaling; partials (max, sum, weighted
// values) go to scratch and are merged per (b,h) in a fixed order.
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kSmThreads = 256;
constexpr int kSmWaves = kSmThreads / 64;
constexpr int kSmRec = kD + 2;          // floats per partial record: o[128], m, l
constexpr int kSmPagesPerBlock = 8;     // page slots per workgroup (one partial record)

template <typename T>
__global__ __launch_bounds__(kSmThreads) void softmax_partial_kernel(
    const T* __restrict__ q, const T* __restrict__ k_pool, const T* __restrict__ v_pool,
    const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ page_idx, const int32_t* __restrict__ n_sel, float* __restrict__ part, int Hq,
    int Hkv, int P, int Mmax, int cap, int n_chunks_max, float scale) {
  __shared__ float s_o[kSmWaves][kD];
  __shared__ float s_m[kSmWaves], s_l[kSmWaves];
  const int bh = blockIdx.y, chunk = blockIdx.x;
  const int b = bh / Hq, hkv = (bh % Hq) / (Hq / Hkv);
  const int n = seq_lens[b];
  const int n_slots = n_sel[bh];
  const int slot0 = chunk * kSmPagesPerBlock;
  if (slot0 >= n_slots) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, r = lane >> 4, c = lane & 15;
  float qv[8];
  load8<T>(q + (size_t)bh * kD + 8 * c, qv);
  float m_run = -INFINITY, l_run = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  constexpr int kPagesPerWave = kSmPagesPerBlock / kSmWaves;
  for (int pw = 0; pw < kPagesPerWave; ++pw) {
    const int slot = slot0 + w * kPagesPerWave + pw;
    if (slot >= n_slots) break;
    const int lp = page_idx[(size_t)bh * cap + slot];
    const int phys = block_table[(size_t)b * Mmax + lp];
    const size_t page_off = ((size_t)phys * Hkv + hkv) * P * kD + 8 * c;
    for (int s = 0; s < P / 4; ++s) {
      const int tok = 4 * s + r;
      float x[8];
      load8<T>(k_pool + page_off + (size_t)tok * kD, x);
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) d = fmaf(qv[i], x[i], d);
      d = row16_sum(d);
      const bool valid = lp * P + tok < n;
      const float sc = valid ? scale * d : -INFINITY;
      float mx = fmaxf(sc, __shfl_xor(sc, 16));
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx);
      if (m_new > -INFINITY) {
        const float resc = __expf(m_run - m_new);          // exp(-inf) = 0 on the first valid step
        const float p = valid ? __expf(sc - m_new) : 0.f;
        l_run = l_run * resc + p;
        float v[8];
        load8<T>(v_pool + page_off + (size_t)tok * kD, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(p, v[i], acc[i] * resc);
        m_run = m_new;
      }
    }
  }
  // rows of the wavefront share m_run; add their partial sums
  l_run += __shfl_xor(l_run, 16); l_run += __shfl_xor(l_run, 32);
#pragma unroll
  for (int i = 0; i < 8; ++i) { acc[i] += __shfl_xor(acc[i], 16); acc[i] += __shfl_xor(acc[i], 32); }
  if (lane < 16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) s_o[w][8 * c + i] = acc[i];
  }
  if (lane == 0) { s_m[w] = m_run; s_l[w] = l_run; }
  __syncthreads();
  if (threadIdx.x < kD) {
    float M = s_m[0];
    for (int i = 1; i < kSmWaves; ++i) M = fmaxf(M, s_m[i]);
    float L = 0.f, o = 0.f;
    for (int i = 0; i < kSmWaves; ++i) {
      const float f = s_m[i] > -INFINITY ? __expf(s_m[i] - M) : 0.f;
      L += s_l[i] * f; o += s_o[i][threadIdx.x] * f;
    }
    float* rec = part + ((size_t)bh * n_chunks_max + chunk) * kSmRec;
    rec[threadIdx.x] = o;
    if (threadIdx.x == 0) { rec[kD] = M; rec[kD + 1] = L; }
  }
}

__global__ __launch_bounds__(kD) void softmax_merge_kernel(const float* __restrict__ part,
                                                           const int32_t* __restrict__ n_sel,
                                                           float* __restrict__ out, float* __restrict__ lse,
                                                           int n_chunks_max) {
  const int bh = blockIdx.x, t = threadIdx.x;
  const int n_chunks = (n_sel[bh] + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  const float* rec0 = part + (size_t)bh * n_chunks_max * kSmRec;
  float M = -INFINITY;
  for (int i = 0; i < n_chunks; ++i) M = fmaxf(M, rec0[(size_t)i * kSmRec + kD]);
  float L = 0.f, o = 0.f;
  for (int i = 0; i < n_chunks; ++i) {
    const float* rec = rec0 + (size_t)i * kSmRec;
    const float f = rec[kD] > -INFINITY ? __expf(rec[kD] - M) : 0.f;
    L += rec[kD + 1] * f; o += rec[t] * f;
  }
  out[(size_t)bh * kD + t] = L > 0.f ? o / L : 0.f;
  if (t == 0) lse[bh] = L > 0.f ? M + __logf(L) : -INFINITY;
}

size_t softmax_ws_bytes(const Dims& dm) {
  const int n_chunks_max = (dm.cap + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  size_t b = (size_t)dm.B * dm.Hq * n_chunks_max * kSmRec * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

void launch_decode_sparse_softmax(const Dims& dm, const void* q, const ekv_cache_view& c,
                                  const int32_t* page_idx, const int32_t* n_sel, float* out, float* lse_sel,
                                  void* ws, hipStream_t st) {
  const int n_chunks_max = (dm.cap + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  dim3 grid(n_chunks_max, dm.B * dm.Hq);
  if (dm.dtype == EKV_F32)
    hipLaunchKernelGGL(softmax_partial_kernel<float>, grid, dim3(kSmThreads), 0, st, (const float*)q,
                       (const float*)c.k_pool, (const float*)c.v_pool, c.block_table, c.seq_lens, page_idx, n_sel,
                       (float*)ws, dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, n_chunks_max, dm.scale);
  else
    hipLaunchKernelGGL(softmax_partial_kernel<bf16_t>, grid, dim3(kSmThreads), 0, st, (const bf16_t*)q,
                       (const bf16_t*)c.k_pool, (const bf16_t*)c.v_pool, c.block_table, c.seq_lens, page_idx,
                       n_sel, (float*)ws, dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, n_chunks_max, dm.scale);
  hipLaunchKernelGGL(softmax_merge_kernel, dim3(dm.B * dm.Hq), dim3(kD), 0, st, (const float*)ws, n_sel, out,
                     lse_sel, n_chunks_max);
}

}  // namespace ekv
