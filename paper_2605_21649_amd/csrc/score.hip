// Query-aware page scoring (paper Sec. 4.2 Eq. 9 and Sec. 4.3 page moments).
//
// The statistics arrays are [B][Hkv][Mmax][2][128] in logical page order, so one (sequence, KV head)
// is a single contiguous stream.  A wavefront step loads two page records (2 x 2 x 128 elements) with
// one 16-byte load per lane and produces the scores of the G query heads that share the KV head:
//   box   = scale * (q+ . k_max + q- . k_min)     (term by term the same products as Eq. 9's max)
//   mu    = scale * q . k_avg ,  sigma = scale * sqrt(q^2 . k_std^2)
// Reductions run inside 16-lane DPP rows; results are staged in LDS and written coalesced.
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kScoreTile = 64;    // pages per workgroup (4 wavefronts x 8 steps x 2 pages)
constexpr int kScoreSteps = kScoreTile / 4 / 2;

template <typename T, int G, bool GAUSS>
__global__ __launch_bounds__(256) void score_pages_kernel(const T* __restrict__ q,
                                                          const T* __restrict__ stats,
                                                          const int32_t* __restrict__ seq_lens,
                                                          float* __restrict__ out0,   // box or mu
                                                          float* __restrict__ out1,   // sigma (GAUSS)
                                                          int Hkv, int P, int Mmax, float scale) {
  __shared__ float stage[2][G][kScoreTile];
  const int b = blockIdx.z, h = blockIdx.y;
  const int tile0 = blockIdx.x * kScoreTile;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int half = lane >> 5, which = (lane >> 4) & 1, c = lane & 15;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const int Hq = Hkv * G;

  // per-lane query coefficients for its 8 channels
  float coef[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float qv[8];
    load8<T>(q + ((size_t)b * Hq + h * G + g) * kD + 8 * c, qv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (GAUSS) coef[g][i] = which ? qv[i] * qv[i] : qv[i];
      else       coef[g][i] = which ? fmaxf(qv[i], 0.f) : fminf(qv[i], 0.f);
    }
  }

  const int pw0 = tile0 + w * (kScoreTile / 4);            // first page of this wavefront
  const T* base = stats + (((size_t)b * Hkv + h) * Mmax) * 2 * kD;
  float x[kScoreSteps][8];
#pragma unroll
  for (int it = 0; it < kScoreSteps; ++it) {
    const int p = pw0 + 2 * it + half;
    if (p < M) load8<T>(base + ((size_t)p * 2 + which) * kD + 8 * c, x[it]);
    else {
#pragma unroll
      for (int i = 0; i < 8; ++i) x[it][i] = 0.f;
    }
  }
#pragma unroll
  for (int it = 0; it < kScoreSteps; ++it) {
    const int pt = w * (kScoreTile / 4) + 2 * it + half;   // page index inside the tile
    if (GAUSS && which) {
#pragma unroll
      for (int i = 0; i < 8; ++i) x[it][i] *= x[it][i];
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc = fmaf(coef[g][i], x[it][i], acc);
      acc = row16_sum(acc);
      if (GAUSS) {
        if (c == 0) stage[which][g][pt] = which ? scale * sqrtf(acc) : scale * acc;
      } else {
        acc += __shfl_xor(acc, 16);
        if (c == 0 && which == 0) stage[0][g][pt] = scale * acc;
      }
    }
  }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * kScoreTile; idx += 256) {
    const int g = idx / kScoreTile, pt = idx - g * kScoreTile;
    const int p = tile0 + pt;
    if (p >= Mmax) continue;
    const size_t o = ((size_t)b * Hq + h * G + g) * Mmax + p;
    const bool valid = p < M;
    out0[o] = valid ? stage[0][g][pt] : -INFINITY;
    if (GAUSS) out1[o] = valid ? stage[1][g][pt] : 0.f;
  }
}

template <typename T, int G>
static void launch_score_T(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                           int mode, float* box, float* mu, float* sigma, hipStream_t st) {
  dim3 grid((dm.Mmax + kScoreTile - 1) / kScoreTile, dm.Hkv, dm.B), block(256);
  if (mode & EKV_SCORE_BOX)
    hipLaunchKernelGGL((score_pages_kernel<T, G, false>), grid, block, 0, st, (const T*)q, (const T*)s.box,
                       seq_lens, box, (float*)nullptr, dm.Hkv, dm.P, dm.Mmax, dm.scale);
  if (mode & EKV_SCORE_GAUSS)
    hipLaunchKernelGGL((score_pages_kernel<T, G, true>), grid, block, 0, st, (const T*)q, (const T*)s.gauss,
                       seq_lens, mu, sigma, dm.Hkv, dm.P, dm.Mmax, dm.scale);
}

template <typename T>
static void launch_score_G(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                           int mode, float* box, float* mu, float* sigma, hipStream_t st) {
  switch (dm.G) {
    case 1: launch_score_T<T, 1>(dm, q, s, seq_lens, mode, box, mu, sigma, st); break;
    case 2: launch_score_T<T, 2>(dm, q, s, seq_lens, mode, box, mu, sigma, st); break;
    case 4: launch_score_T<T, 4>(dm, q, s, seq_lens, mode, box, mu, sigma, st); break;
    default: launch_score_T<T, 8>(dm, q, s, seq_lens, mode, box, mu, sigma, st); break;
  }
}

void launch_score_pages(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                        int mode, float* box, float* mu, float* sigma, hipStream_t st) {
  if (dm.dtype == EKV_F32) launch_score_G<float>(dm, q, s, seq_lens, mode, box, mu, sigma, st);
  else launch_score_G<bf16_t>(dm, q, s, seq_lens, mode, box, mu, sigma, st);
}

}  // namespace ekv
