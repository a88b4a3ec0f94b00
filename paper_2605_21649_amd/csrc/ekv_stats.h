// Single-page statistics and the token append, shared by the append kernel and by the scoring kernels'
// fused append (paper Sec. 4.2).
#pragma once
#include "ekv_device.h"

namespace ekv {

// Single-page layout (the append): one wavefront per page, lane = (row mod 4, channel group); the four
// partial sums live in the four DPP rows and meet in two exchange steps.  If ov_row != nullptr, token
// `ov_slot` takes its values from ov_row[128] instead of the cache (the token being appended).
template <typename T, int PT>   // PT = compile-time page size (all row loads issued as one batch), 0 = runtime
__device__ __forceinline__ void page_stats_wave(const T* __restrict__ kpage, int cnt, int P_rt,
                                                const T* __restrict__ ov_row, int ov_slot,
                                                T* __restrict__ box_out, T* __restrict__ gauss_out,
                                                uint8_t* __restrict__ box8_out) {
  const int P = PT ? PT : P_rt;
  const int lane = threadIdx.x & 63;
  const int r = lane >> 4, c = lane & 15;
  float k0[8];
  load8<T>((ov_row != nullptr && ov_slot == 0 ? ov_row : kpage) + 8 * c, k0);
  float mn[8], mx[8], s1[8], s2[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { mn[i] = INFINITY; mx[i] = -INFINITY; s1[i] = 0.f; s2[i] = 0.f; }
  // rows past cnt re-read row 0 (loads stay unconditional) and are masked out of every statistic
  auto accumulate = [&](const float (&x)[8], bool ok) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      mn[i] = fminf(mn[i], ok ? x[i] : INFINITY);
      mx[i] = fmaxf(mx[i], ok ? x[i] : -INFINITY);
      const float dx = ok ? x[i] - k0[i] : 0.f;
      s1[i] += dx;
      s2[i] = fmaf(dx, dx, s2[i]);
    }
  };
  if constexpr (PT != 0) {
    // the whole page in flight at once, kept in storage format until it is consumed (registers: this
    // function also runs inside the scoring kernels, whose occupancy its register count would set)
    Raw8<T> raw[PT / 4];
#pragma unroll
    for (int s = 0; s < PT / 4; ++s) {
      const int row = 4 * s + r;
      const int rc = row < cnt ? row : 0;
      load_raw8((ov_row != nullptr && rc == ov_slot ? ov_row : kpage + (size_t)rc * kD) + 8 * c, raw[s]);
    }
#pragma unroll
    for (int s = 0; s < PT / 4; ++s) {
      float x[8];
      widen8(raw[s], x);
      accumulate(x, 4 * s + r < cnt);
    }
  } else {
    for (int t0 = 0; t0 < P; t0 += kRowsPerWave) {
      const int row = t0 + r;
      const int rc = row < cnt ? row : 0;
      float x[8];
      load8<T>((ov_row != nullptr && rc == ov_slot ? ov_row : kpage + (size_t)rc * kD) + 8 * c, x);
      accumulate(x, row < cnt);
    }
  }
  const float inv_n = 1.0f / (float)cnt;
  float avg[8], sd[8];   // sd holds the variance m2 - avg^2 (clamped at 0)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    mn[i] = fminf(mn[i], __shfl_xor(mn[i], 16)); mn[i] = fminf(mn[i], __shfl_xor(mn[i], 32));
    mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 16)); mx[i] = fmaxf(mx[i], __shfl_xor(mx[i], 32));
    s1[i] += __shfl_xor(s1[i], 16); s1[i] += __shfl_xor(s1[i], 32);
    s2[i] += __shfl_xor(s2[i], 16); s2[i] += __shfl_xor(s2[i], 32);
    const float m1 = s1[i] * inv_n;
    const float var = fmaxf(fmaf(-m1, m1, s2[i] * inv_n), 0.f);
    avg[i] = k0[i] + m1;
    sd[i] = var;
  }
  if (r == 0) {
    store8<T>(box_out + 8 * c, mn);
    store8<T>(box_out + kD + 8 * c, mx);
    store8<T>(gauss_out + 8 * c, avg);
    store8<T>(gauss_out + kD + 8 * c, sd);
    if (box8_out != nullptr) store_box8_unit(box8_out + 16 * c, mn, mx);
  }
}

// Appends one token to (sequence b, KV head h) with ONE wavefront (lane = threadIdx.x & 63): writes k_new
// (and v_new) into slot `pos` of the cache and recomputes the statistics of that page over its pos%P + 1
// tokens.  Nothing happens when the page is not mapped (pos < 0 or pos/P >= Mmax).
template <typename T, int PT>
__device__ __forceinline__ void append_token_wave(T* __restrict__ k_pool, T* __restrict__ v_pool,
                                                  const int32_t* __restrict__ block_table, int pos,
                                                  const T* __restrict__ k_new, const T* __restrict__ v_new,
                                                  T* __restrict__ box, T* __restrict__ gauss,
                                                  uint8_t* __restrict__ box8, int b, int h, int Hkv,
                                                  int HkvPool, int P, int Mmax, int n_phys) {
  const int p = pos / P, slot = pos - p * P;
  if (pos < 0 || p >= Mmax) return;            // no room: validated against on the host where possible
  const int phys = min(max(block_table[(size_t)b * Mmax + p], 0), n_phys - 1);
  const size_t page_off = ((size_t)phys * HkvPool + h) * P * kD;
  const T* knew = k_new + ((size_t)b * Hkv + h) * kD;
  const int lane = threadIdx.x & 63;
  if (lane < 16) {
    float x[8];
    load8<T>(knew + 8 * lane, x);
    store8<T>(k_pool + page_off + (size_t)slot * kD + 8 * lane, x);
  } else if (lane < 32 && v_new != nullptr) {
    float x[8];
    const int c = lane - 16;
    load8<T>(v_new + ((size_t)b * Hkv + h) * kD + 8 * c, x);
    store8<T>(v_pool + page_off + (size_t)slot * kD + 8 * c, x);
  }
  const size_t rec = (((size_t)b * Hkv + h) * Mmax + p) * 2 * kD;
  page_stats_wave<T, PT>(k_pool + page_off, slot + 1, P, knew, slot, box + rec, gauss + rec,
                         box8 != nullptr ? box8 + rec : nullptr);       // 256 bytes per page in either array
}

}  // namespace ekv
