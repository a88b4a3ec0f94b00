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

// One wavefront handles kSmPagesPerBlock / kSmWaves pages; the K and V rows of a page are fetched as one
// batch of unconditional loads (lane = (token mod 4, channel group)), the running maximum is updated once
// per page.  Page and block-table indices are clamped into range; tokens past the sequence end are masked.
// Work distribution: an item is one chunk of kSmPagesPerBlock page slots of one (b,h) row.  The launch has a fixed
// number of workgroups that does not depend on the capacity of the page lists: every workgroup builds the exclusive
// prefix of the chunks per row from the device-side list lengths (LDS) and takes a contiguous range of the
// concatenated chunks.  (Launches with more rows than LDS holds fall back to one workgroup per chunk of capacity.)
struct SmArgs {
  const void* q; const void* k_pool; const void* v_pool;
  const int32_t* block_table; const int32_t* seq_lens; const int32_t* page_idx; const int32_t* n_sel;
  float* part;
  int rows, Hq, Hkv, HkvPool, P_rt, Mmax, cap, n_chunks_max, n_phys;
  float scale;
};
constexpr int kSmRowsLdsMax = 8192;

template <typename T, int PT>   // PT = compile-time page size (16 or 32), 0 = runtime
__device__ __forceinline__ void softmax_chunk(const SmArgs& A, int bh, int chunk, float (&s_o)[kSmWaves][kD],
                                              float (&s_m)[kSmWaves], float (&s_l)[kSmWaves]) {
  const T* q = (const T*)A.q;
  const T* k_pool = (const T*)A.k_pool;
  const T* v_pool = (const T*)A.v_pool;
  constexpr int kPagesPerWave = kSmPagesPerBlock / kSmWaves;
  constexpr int SMAX = PT ? PT / 4 : 16;            // row steps per page (page size <= 64)
  const int P = PT ? PT : A.P_rt;
  const int Hq = A.Hq, Hkv = A.Hkv, cap = A.cap, Mmax = A.Mmax;
  const int b = bh / Hq, hkv = (bh % Hq) / (Hq / Hkv);
  const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int r = lane >> 4, c = lane & 15;
  const int slot0 = chunk * kSmPagesPerBlock;
  const int wslot0 = slot0 + w * kPagesPerWave;
  int lps[kPagesPerWave], physs[kPagesPerWave];
#pragma unroll
  for (int i = 0; i < kPagesPerWave; ++i)
    lps[i] = min(max(A.page_idx[(size_t)bh * cap + min(wslot0 + i, cap - 1)], 0), Mmax - 1);
  const int n = A.seq_lens[b];
  const int n_slots = min(max(A.n_sel[bh], 0), cap);
#pragma unroll
  for (int i = 0; i < kPagesPerWave; ++i)
    physs[i] = min(max(A.block_table[(size_t)b * Mmax + lps[i]], 0), A.n_phys - 1);
  float qv[8];
  load8<T>(q + (size_t)bh * kD + 8 * c, qv);
  float m_run = -INFINITY, l_run = 0.f, acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
#pragma unroll
  for (int pw = 0; pw < kPagesPerWave; ++pw) {
    const bool slot_ok = wslot0 + pw < n_slots;      // wave-uniform
    const size_t page_off = ((size_t)physs[pw] * A.HkvPool + hkv) * P * kD + 8 * c;
    const int steps = P / 4;
    Raw8<T> kr[SMAX], vr[SMAX];
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
      const int tok = 4 * min(s, steps - 1) + r;
      load_raw8(k_pool + page_off + (size_t)tok * kD, kr[s]);
      load_raw8(v_pool + page_off + (size_t)tok * kD, vr[s]);
    }
    float sc[SMAX];
    float mx = -INFINITY;
#pragma unroll
    for (int s = 0; s < SMAX; ++s) {
      float x[8];
      widen8(kr[s], x);
      float d = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) d = fmaf(qv[i], x[i], d);
      d = row16_sum(d);
      const bool valid = slot_ok && s < steps && lps[pw] * P + 4 * s + r < n;
      sc[s] = valid ? A.scale * d : -INFINITY;
      mx = fmaxf(mx, sc[s]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    if (m_new > -INFINITY) {                          // wave-uniform; no loads inside
      const float resc = __expf(m_run - m_new);      // exp(-inf) = 0 on the first valid page
      l_run *= resc;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] *= resc;
#pragma unroll
      for (int s = 0; s < SMAX; ++s) {
        const float p = __expf(sc[s] - m_new);       // 0 for masked tokens
        l_run += p;
        float v[8];
        widen8(vr[s], v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(p, v[i], acc[i]);
      }
      m_run = m_new;
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
    float* rec = A.part + ((size_t)bh * A.n_chunks_max + chunk) * kSmRec;
    rec[threadIdx.x] = o;
    if (threadIdx.x == 0) { rec[kD] = M; rec[kD + 1] = L; }
  }
}

template <typename T, int PT, bool CAP_GRID>
__global__ __launch_bounds__(kSmThreads) void softmax_partial_kernel(const SmArgs A) {
  __shared__ float s_o[kSmWaves][kD];
  __shared__ float s_m[kSmWaves], s_l[kSmWaves];
  extern __shared__ int sm_pre[];                   // [rows + 1] chunks per row, exclusive prefix
  __shared__ int wsum[kSmWaves];
  if (CAP_GRID) {                                   // one workgroup per chunk of capacity
    const int bh = blockIdx.y, chunk = blockIdx.x;
    if (chunk * kSmPagesPerBlock >= min(max(A.n_sel[bh], 0), A.cap)) return;     // workgroup-uniform
    softmax_chunk<T, PT>(A, bh, chunk, s_o, s_m, s_l);
    return;
  }
  block_exclusive_prefix<kSmThreads>(A.rows, [&](int u) {
    return (min(max(A.n_sel[u], 0), A.cap) + kSmPagesPerBlock - 1) / kSmPagesPerBlock; }, sm_pre, wsum);
  const int total = sm_pre[A.rows];
  const int G = gridDim.x, wg = blockIdx.x;
  const int per = total / G, rem = total - per * G;
  const int begin = wg * per + min(wg, rem), end = begin + per + (wg < rem ? 1 : 0);
  if (begin >= end) return;
  int lo = 0, hi = A.rows;                          // sm_pre[lo] <= begin < sm_pre[hi]
  while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (sm_pre[mid] <= begin) lo = mid; else hi = mid; }
  int bh = lo;
  for (int it = begin; it < end; ++it) {
    while (it >= sm_pre[bh + 1]) ++bh;
    softmax_chunk<T, PT>(A, bh, it - sm_pre[bh], s_o, s_m, s_l);
    __syncthreads();                                // the LDS partials are reused by the next chunk
  }
}

// Merge of the per-chunk partials of one (b,h): 8 groups of 128 threads take the chunks round robin
// (independent loads), then the groups are combined through LDS in index order.
constexpr int kMergeGroups = 8;
__global__ __launch_bounds__(kMergeGroups * kD) void softmax_merge_kernel(const float* __restrict__ part,
                                                                          const int32_t* __restrict__ n_sel,
                                                                          float* __restrict__ out,
                                                                          float* __restrict__ lse,
                                                                          int n_chunks_max, int cap) {
  __shared__ float red[kMergeGroups * kD / 64];
  __shared__ float g_o[kMergeGroups][kD], g_l[kMergeGroups];
  const int bh = blockIdx.x, tid = threadIdx.x, t = tid & (kD - 1), grp = tid >> 7;
  const int n_chunks = (min(max(n_sel[bh], 0), cap) + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  const float* rec0 = part + (size_t)bh * n_chunks_max * kSmRec;
  float mx = -INFINITY;
  for (int i = tid; i < n_chunks; i += kMergeGroups * kD) mx = fmaxf(mx, rec0[(size_t)i * kSmRec + kD]);
  const float M = block_max(mx, red);
  float L = 0.f, o = 0.f;
  for (int i0 = grp; i0 < n_chunks; i0 += 4 * kMergeGroups) {
    float rm[4], rl[4], ro[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float* rec = rec0 + (size_t)min(i0 + u * kMergeGroups, n_chunks - 1) * kSmRec;
      rm[u] = rec[kD]; rl[u] = rec[kD + 1]; ro[u] = rec[t];
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float f = (i0 + u * kMergeGroups < n_chunks && rm[u] > -INFINITY) ? __expf(rm[u] - M) : 0.f;
      L += rl[u] * f; o += ro[u] * f;
    }
  }
  g_o[grp][t] = o;
  if (t == 0) g_l[grp] = L;
  __syncthreads();
  if (tid < kD) {
    float Ls = 0.f, os = 0.f;
    for (int g = 0; g < kMergeGroups; ++g) { Ls += g_l[g]; os += g_o[g][tid]; }
    out[(size_t)bh * kD + tid] = Ls > 0.f ? os / Ls : 0.f;
    if (tid == 0) lse[bh] = Ls > 0.f ? M + __logf(Ls) : -INFINITY;
  }
}

size_t softmax_ws_bytes(const Dims& dm) {
  const int n_chunks_max = (dm.cap + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  size_t b = (size_t)dm.B * dm.Hq * n_chunks_max * kSmRec * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

static int sm_compute_units() {
  int dev = 0, n = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
  return n;
}

template <typename T>
static void launch_softmax_T(const Dims& dm, const void* q, const ekv_cache_view& c, const int32_t* page_idx,
                             const int32_t* n_sel, float* ws, int n_chunks_max, hipStream_t st) {
  const int rows = dm.B * dm.Hq;
  SmArgs sa{q, c.k_pool, c.v_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws,
            rows, dm.Hq, dm.Hkv, dm.HkvPool, dm.P, dm.Mmax, dm.cap, n_chunks_max, c.n_phys_pages, dm.scale};
  dim3 block(kSmThreads);
  if (rows > kSmRowsLdsMax) {
    dim3 grid(n_chunks_max, rows);
#define EKV_SM(PT) hipLaunchKernelGGL((softmax_partial_kernel<T, PT, true>), grid, block, 0, st, sa)
    if (dm.P == 16) EKV_SM(16); else if (dm.P == 32) EKV_SM(32); else EKV_SM(0);
#undef EKV_SM
    return;
  }
  // a fixed grid (16 workgroups per compute unit, never more than the lists can hold chunks)
  long long wgs = (long long)rows * n_chunks_max;
  const long long wg_cap = (long long)sm_compute_units() * 16;
  if (wgs > wg_cap) wgs = wg_cap;
  if (wgs < 1) wgs = 1;
  dim3 grid((unsigned)wgs);
  const size_t lds = (size_t)(rows + 1) * sizeof(int);
#define EKV_SM(PT) hipLaunchKernelGGL((softmax_partial_kernel<T, PT, false>), grid, block, lds, st, sa)
  if (dm.P == 16) EKV_SM(16); else if (dm.P == 32) EKV_SM(32); else EKV_SM(0);
#undef EKV_SM
}

void launch_decode_sparse_softmax(const Dims& dm, const void* q, const ekv_cache_view& c,
                                  const int32_t* page_idx, const int32_t* n_sel, float* out, float* lse_sel,
                                  void* ws, hipStream_t st) {
  const int n_chunks_max = (dm.cap + kSmPagesPerBlock - 1) / kSmPagesPerBlock;
  if (dm.dtype == EKV_F32) launch_softmax_T<float>(dm, q, c, page_idx, n_sel, (float*)ws, n_chunks_max, st);
  else launch_softmax_T<bf16_t>(dm, q, c, page_idx, n_sel, (float*)ws, n_chunks_max, st);
  hipLaunchKernelGGL(softmax_merge_kernel, dim3(dm.B * dm.Hq), dim3(kMergeGroups * kD), 0, st, (const float*)ws, n_sel,
                     out, lse_sel, n_chunks_max, dm.cap);
}

}  // namespace ekv
