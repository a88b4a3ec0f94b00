// Page-statistics builder (paper Sec. 4.2): per page k_min, k_max, k_avg and k_var = k_std^2
// (the variance is what is stored: sigma_p^2 of Sec. 4.3 is linear in it).
// Sixteen lanes own one page: lane c holds channels 8c..8c+7 and walks the page's rows itself, so no
// statistic ever crosses lanes; a wavefront covers four pages, each row load being four 256-byte
// segments.  The kernel is a stream over K (HBM-bound once the per-element work is this small: min,
// max, subtract, add, fused multiply-add).
#include "ekv_device.h"
#include "ekv_internal.h"
#include "ekv_stats.h"

namespace ekv {

constexpr int kStatRowBatch = 4;     // row loads in flight per lane in the bulk build

// Summation order shared by both layouts below (so that append-then-query equals rebuild-then-query bit
// for bit): rows are split by t mod 4 into four partial sums, each taken in ascending row order relative
// to the first token's value (so that m2 - avg^2 does not cancel for channels with a large common
// offset), combined as (p0 + p1) + (p2 + p3).  Rows past cnt add exact zeros.

// Bulk layout: the 16 lanes of a DPP row own one page; lane c holds channels 8c..8c+7 and walks the
// page's rows itself, so no statistic crosses lanes; a wavefront covers four pages, each row load being
// four 256-byte segments.  `kpage` points at the page's [P][128] block; tokens [0,cnt) are valid.
template <typename T, int PT>   // PT = compile-time page size, 0 = runtime
__device__ __forceinline__ void page_stats_rows(const T* __restrict__ kpage, int cnt, int P_rt, bool all_full,
                                                T* __restrict__ box_out, T* __restrict__ gauss_out,
                                                uint8_t* __restrict__ box8_out) {
  constexpr int RB = kStatRowBatch;
  static_assert(RB == 4, "one batch = one row of each partial sum");
  const int P = PT ? PT : P_rt;
  const int c = threadIdx.x & 15;
  float k0[8];
  load8<T>(kpage + 8 * c, k0);
  float mn[8], mx[8], s1[4][8], s2[4][8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = INFINITY; mx[i] = -INFINITY;
#pragma unroll
    for (int r = 0; r < 4; ++r) { s1[r][i] = 0.f; s2[r][i] = 0.f; }
  }
  if (all_full) {                                        // wave-uniform: every page of the wavefront is full
#pragma unroll 1
    for (int t0 = 0; t0 < P; t0 += RB) {
      Raw8<T> raw[RB];
#pragma unroll
      for (int j = 0; j < RB; ++j) load_raw8(kpage + (size_t)(t0 + j) * kD + 8 * c, raw[j]);   // P % 4 == 0
#pragma unroll
      for (int j = 0; j < RB; ++j) {
        float x[8];
        widen8(raw[j], x);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          mn[i] = fminf(mn[i], x[i]);
          mx[i] = fmaxf(mx[i], x[i]);
          const float dx = x[i] - k0[i];
          s1[j][i] += dx;
          s2[j][i] = fmaf(dx, dx, s2[j][i]);
        }
      }
    }
  } else {
#pragma unroll 1
    for (int t0 = 0; t0 < P; t0 += RB) {
      Raw8<T> raw[RB];
#pragma unroll
      for (int j = 0; j < RB; ++j)                       // rows past cnt re-read row 0: loads stay unconditional
        load_raw8(kpage + (size_t)(t0 + j < cnt ? t0 + j : 0) * kD + 8 * c, raw[j]);
#pragma unroll
      for (int j = 0; j < RB; ++j) {
        const bool ok = t0 + j < cnt;
        float x[8];
        widen8(raw[j], x);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          mn[i] = fminf(mn[i], ok ? x[i] : INFINITY);
          mx[i] = fmaxf(mx[i], ok ? x[i] : -INFINITY);
          const float dx = ok ? x[i] - k0[i] : 0.f;
          s1[j][i] += dx;
          s2[j][i] = fmaf(dx, dx, s2[j][i]);
        }
      }
    }
  }
  const float inv_n = 1.0f / (float)cnt;
  float avg[8], var[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const float t1 = (s1[0][i] + s1[1][i]) + (s1[2][i] + s1[3][i]);
    const float t2 = (s2[0][i] + s2[1][i]) + (s2[2][i] + s2[3][i]);
    const float m1 = t1 * inv_n;
    var[i] = fmaxf(fmaf(-m1, m1, t2 * inv_n), 0.f);      // m2 - avg^2, clamped at 0
    avg[i] = k0[i] + m1;
  }
  store8<T>(box_out + 8 * c, mn);
  store8<T>(box_out + kD + 8 * c, mx);
  store8<T>(gauss_out + 8 * c, avg);
  store8<T>(gauss_out + kD + 8 * c, var);
  if (box8_out != nullptr) store_box8_unit(box8_out + 16 * c, mn, mx);
}

template <typename T, int PT>
__global__ __launch_bounds__(256) void stats_build_kernel(const T* __restrict__ k_pool,
                                                          const int32_t* __restrict__ block_table,
                                                          const int32_t* __restrict__ seq_lens,
                                                          T* __restrict__ box, T* __restrict__ gauss,
                                                          uint8_t* __restrict__ box8,
                                                          int Hkv, int HkvPool, int P, int Mmax, int n_phys) {
  const int b = blockIdx.z, h = blockIdx.y;
  const int p = blockIdx.x * 16 + (threadIdx.x >> 4);     // 16 pages per workgroup, 4 per wavefront
  const int n = seq_lens[b];
  const int M = min((n + P - 1) / P, Mmax);
  const int pc = min(p, M - 1);                           // lanes past the end recompute the last page, unwritten
  if (M <= 0) return;
  const int cnt = min(P, n - pc * P);
  const int phys = min(max(block_table[(size_t)b * Mmax + pc], 0), n_phys - 1);
  const T* kpage = k_pool + ((size_t)phys * HkvPool + h) * P * kD;
  const size_t rec = (((size_t)b * Hkv + h) * Mmax + pc) * 2 * kD;
  const bool all_full = __all(cnt == P);
  if (blockIdx.x * 16 + (int)(threadIdx.x >> 6) * 4 >= M) return;      // whole wavefront past the end
  if (p < M) page_stats_rows<T, PT>(kpage, cnt, P, all_full, box + rec, gauss + rec,
                                    box8 != nullptr ? box8 + rec : nullptr);   // 256 bytes per page there
}

// One wavefront per (sequence, KV head): write the new token into slot n_b and refresh its page.
template <typename T, int PT>
__global__ __launch_bounds__(64) void stats_append_kernel(T* __restrict__ k_pool, T* __restrict__ v_pool,
                                                          const int32_t* __restrict__ block_table,
                                                          const int32_t* __restrict__ seq_lens,
                                                          const T* __restrict__ k_new,
                                                          const T* __restrict__ v_new,
                                                          T* __restrict__ box, T* __restrict__ gauss,
                                                          uint8_t* __restrict__ box8,
                                                          int Hkv, int HkvPool, int P, int Mmax, int n_phys) {
  append_token_wave<T, PT>(k_pool, v_pool, block_table, seq_lens[blockIdx.y], k_new, v_new, box, gauss, box8,
                           blockIdx.y, blockIdx.x, Hkv, HkvPool, P, Mmax, n_phys);
}

template <typename T, int PT>
static void launch_build_T(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s, hipStream_t st) {
  dim3 grid((dm.Mmax + 15) / 16, dm.Hkv, dm.B), block(256);
  hipLaunchKernelGGL((stats_build_kernel<T, PT>), grid, block, 0, st, (const T*)c.k_pool, c.block_table, c.seq_lens,
                     (T*)s.box, (T*)s.gauss, (uint8_t*)s.box8, dm.Hkv, dm.HkvPool, dm.P, dm.Mmax, c.n_phys_pages);
}
template <typename T, int PT>
static void launch_append_T(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s, const void* k_new,
                            const void* v_new, hipStream_t st) {
  dim3 grid(dm.Hkv, dm.B), block(64);
  hipLaunchKernelGGL((stats_append_kernel<T, PT>), grid, block, 0, st, (T*)c.k_pool, (T*)c.v_pool, c.block_table,
                     c.seq_lens, (const T*)k_new, (const T*)v_new, (T*)s.box, (T*)s.gauss, (uint8_t*)s.box8, dm.Hkv,
                     dm.HkvPool, dm.P, dm.Mmax, c.n_phys_pages);
}

void launch_stats_build(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s, hipStream_t st) {
  const bool f32 = dm.dtype == EKV_F32;
  if (dm.P == 16) { if (f32) launch_build_T<float, 16>(dm, c, s, st); else launch_build_T<bf16_t, 16>(dm, c, s, st); }
  else if (dm.P == 32) { if (f32) launch_build_T<float, 32>(dm, c, s, st); else launch_build_T<bf16_t, 32>(dm, c, s, st); }
  else { if (f32) launch_build_T<float, 0>(dm, c, s, st); else launch_build_T<bf16_t, 0>(dm, c, s, st); }
}

void launch_stats_append(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s,
                         const void* k_new, const void* v_new, hipStream_t st) {
  const bool f32 = dm.dtype == EKV_F32;
  if (dm.P == 16) { if (f32) launch_append_T<float, 16>(dm, c, s, k_new, v_new, st); else launch_append_T<bf16_t, 16>(dm, c, s, k_new, v_new, st); }
  else if (dm.P == 32) { if (f32) launch_append_T<float, 32>(dm, c, s, k_new, v_new, st); else launch_append_T<bf16_t, 32>(dm, c, s, k_new, v_new, st); }
  else if (dm.P == 64) { if (f32) launch_append_T<float, 64>(dm, c, s, k_new, v_new, st); else launch_append_T<bf16_t, 64>(dm, c, s, k_new, v_new, st); }
  else { if (f32) launch_append_T<float, 0>(dm, c, s, k_new, v_new, st); else launch_append_T<bf16_t, 0>(dm, c, s, k_new, v_new, st); }
}

}  // namespace ekv
