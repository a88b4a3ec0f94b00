// Query-aware page scoring (paper Sec. 4.2 Eq. 9 and Sec. 4.3 page moments).
//
// The statistics arrays are [B][Hkv][Mmax][2][128] in logical page order, so one (sequence, KV head)
// is a single contiguous stream.  Per page the kernel needs, for the G query heads of the group,
//   box    = scale * (q- . k_min + q+ . k_max)       (term by term the same products as Eq. 9's max)
//   mu     = scale * q . k_avg ,   sigma = scale * sqrt(q^2 . k_var)         (k_var = k_std^2)
// i.e. a [pages x 256] x [256 x G] contraction.  bf16 statistics go through the matrix cores
// (v_mfma_f32_16x16x32_bf16): an MFMA tile holds 4 pages x 4 channel quarters as its 16 rows and
// G heads x 4 channel quarters as its 16 columns, so that every lane's A operand is the 16 bytes of a
// fully coalesced load; only the blocks with matching quarters are meaningful and are summed with
// two DPP quad steps.  q^2 is split exactly into two bf16 values (a product of two 8-bit significands
// has 16 bits).  float32 statistics use plain FMAs and DPP row reductions.
// With EKV_SCORE_GROUP_MAX the box scores of the G heads are reduced to their maximum before they are
// written (one list of pages per KV head, shared by its query heads).
#include "ekv_device.h"
#include "ekv_internal.h"
#include "ekv_stats.h"

namespace ekv {

// Pages per workgroup: 4 wavefronts x 8 pages (16 KiB of statistics).  Measured at 1M tokens: 46.5 us per launch,
// 47.7 with 64 pages, 52 with 128 -- small workgroups at high occupancy keep more of the stream in flight.
constexpr int kScoreTile = 32;

// Fused append: the workgroup that scores the tile holding the page of the new token first appends it (one
// wavefront: cache slot written, page statistics recomputed); every workgroup scores with the length n_b + 1.
// mode 0: plain scoring; 1: append, then score; 2: score with n_b + 1 only (a second launch of the call).
struct ScoreAppend {
  void* k_pool; void* v_pool; const int32_t* block_table; const void* k_new; const void* v_new;
  void* box_stats; void* gauss_stats; void* box8_stats;
  int n_phys, mode, hkv_pool;
  int units, n_tiles;     // (sequence, KV head) units and tiles per unit of this launch
};

// What a workgroup does.  The grid is one-dimensional (folded over x and y): workgroup j scores tile
// j % n_tiles of unit j / n_tiles -- tile index fastest, so that consecutive workgroups read consecutive
// parts of one unit's statistics stream.  A launch that appends puts one extra workgroup per unit IN FRONT
// of all of those: it appends the unit's token and scores the tile of that page, and the regular workgroup of
// that tile leaves at once.  The appending workgroups are then the first ones dispatched and their extra
// latency hides behind the stream (as part of the regular order, the last unit's started near the end of
// the launch and lengthened it by 2 us).
struct TileWork { int b, h, tile0, n; bool run; };

// APPEND = false instantiations carry no append code at all (modes 0 and 2): their register count, and with it
// the occupancy of the stream, is that of the scoring loop alone.
template <typename T, bool APPEND>
__device__ __forceinline__ TileWork score_work(const ScoreAppend& ap, const int32_t* __restrict__ seq_lens, int Hkv,
                                               int P, int Mmax, int tile) {
  TileWork tw{0, 0, 0, 0, false};
  const bool appending = APPEND && ap.mode == 1;
  const long long gid = (long long)blockIdx.y * gridDim.x + blockIdx.x;
  const long long total = (long long)ap.units * ap.n_tiles + (appending ? ap.units : 0);
  if (gid >= total) return tw;
  const bool front = appending && gid < ap.units;
  int unit, tix;
  if (front) { unit = (int)gid; tix = 0; }
  else if (total <= 0x7fffffffLL) {                 // the usual case: 32-bit division
    const int j = (int)(appending ? gid - ap.units : gid);
    unit = j / ap.n_tiles; tix = j - unit * ap.n_tiles;
  } else {
    const long long j = appending ? gid - ap.units : gid;
    unit = (int)(j / ap.n_tiles); tix = (int)(j - (long long)unit * ap.n_tiles);
  }
  tw.b = unit / Hkv; tw.h = unit - tw.b * Hkv;
  const int n = seq_lens[tw.b];
  const int p_new = n / P;
  const bool has_new = ap.mode != 0 && n >= 0 && p_new < Mmax;      // false: no room, nothing is appended
  tw.n = has_new ? n + 1 : n;
  if (appending) {
    const int t_new = p_new / tile;
    if (front) {
      if (!has_new) return tw;
      tix = t_new;
      if (threadIdx.x < 64) {
        // 16-token pages fetch the whole page as one batch (as the append kernel does); other sizes take the
        // row-by-row instantiation, same summation order, because the register count of this path sets the
        // occupancy of every streaming workgroup of the launch
        if (P == 16)
          append_token_wave<T, 16>((T*)ap.k_pool, (T*)ap.v_pool, ap.block_table, n, (const T*)ap.k_new,
                                   (const T*)ap.v_new, (T*)ap.box_stats, (T*)ap.gauss_stats, (uint8_t*)ap.box8_stats,
                                   tw.b, tw.h, Hkv, ap.hkv_pool, P, Mmax, ap.n_phys);
        else
          append_token_wave<T, 0>((T*)ap.k_pool, (T*)ap.v_pool, ap.block_table, n, (const T*)ap.k_new,
                                  (const T*)ap.v_new, (T*)ap.box_stats, (T*)ap.gauss_stats, (uint8_t*)ap.box8_stats,
                                  tw.b, tw.h, Hkv, ap.hkv_pool, P, Mmax, ap.n_phys);
      }
      // the statistics rows written above are read below by the other wavefronts of this workgroup only (same
      // compute unit): a workgroup-scope fence is enough; a device-scope one would write back the whole L2
      __threadfence_block();
      __syncthreads();
    } else if (has_new && tix == t_new) {
      return tw;                                       // scored by the appending workgroup
    }
  }
  tw.tile0 = tix * tile;
  tw.run = true;
  return tw;
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

__device__ __forceinline__ f32x4_t mfma_bf16(const uint4& a, const uint4& b, f32x4_t c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b),
                                                 c, 0, 0, 0);
}

// keep the negative (NEG) or the non-negative bf16 halves of a packed pair, zero the others
template <bool NEG> __device__ __forceinline__ uint32_t keep_sign(uint32_t x) {
  const uint32_t lo_neg = (x & 0x00008000u) ? 0x0000ffffu : 0u;
  const uint32_t hi_neg = (x & 0x80000000u) ? 0xffff0000u : 0u;
  const uint32_t m = lo_neg | hi_neg;
  return NEG ? (x & m) : (x & ~m);
}

// q^2 of a packed bf16 pair, split exactly into hi + lo bf16 parts (truncation keeps the top 8 bits of
// the 16-bit product; the remainder has at most 8 significant bits)
__device__ __forceinline__ void square_split(uint32_t x, uint32_t& hi, uint32_t& lo) {
  const float a = __uint_as_float(x << 16), b = __uint_as_float(x & 0xffff0000u);
  const float a2 = a * a, b2 = b * b;
  const uint32_t a_hi = __float_as_uint(a2) & 0xffff0000u, b_hi = __float_as_uint(b2) & 0xffff0000u;
  const float a_lo = a2 - __uint_as_float(a_hi), b_lo = b2 - __uint_as_float(b_hi);
  hi = (a_hi >> 16) | b_hi;
  lo = (__float_as_uint(a_lo) >> 16) | (__float_as_uint(b_lo) & 0xffff0000u);
}

// The meaningful entry of an MFMA result for this lane (the block whose row quarter equals the column
// quarter kq = lane & 3), summed over the four quarters held by the lanes of a quad.
__device__ __forceinline__ float diag_quad_sum(const f32x4_t& c, int kq) {
  float v = kq == 0 ? c[0] : kq == 1 ? c[1] : kq == 2 ? c[2] : c[3];
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  return v;
}

// Eight E4M3 codes (two dwords) -> eight bf16 values (exact: every E4M3 value is a bf16 value).
__device__ __forceinline__ uint4 e4m3x8_to_bf16x8(uint32_t lo, uint32_t hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  uint4 r;
  r.x = __builtin_bit_cast(uint32_t, (bf16x2_t)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, false));
  r.y = __builtin_bit_cast(uint32_t, (bf16x2_t)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(lo, 1.0f, true));
  r.z = __builtin_bit_cast(uint32_t, (bf16x2_t)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, false));
  r.w = __builtin_bit_cast(uint32_t, (bf16x2_t)__builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(hi, 1.0f, true));
  return r;
}

enum : int { kKindBox = 0, kKindGauss = 1, kKindBox8 = 2 };
// pages per workgroup: 4 wavefronts x 8 pages of 512-byte records, or x 16 pages of 256-byte 8-bit records
// (the same bytes per wavefront)
__host__ __device__ constexpr int score_tile(int kind) { return kind == kKindBox8 ? 2 * kScoreTile : kScoreTile; }

// At least six wavefronts per SIMD: the scoring loop needs about 45 registers, the fused append path about 90, and
// the stream is faster with the append squeezed (a few spilled values in its one wavefront) than with every
// workgroup of the launch at an occupancy of four.
template <int G, int KIND, bool APPEND>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(6, 8)))
void score_pages_mfma_kernel(const bf16_t* __restrict__ q,
                                                               const void* __restrict__ stats_any,
                                                               const int32_t* __restrict__ seq_lens,
                                                               float* __restrict__ out0,   // box or mu
                                                               float* __restrict__ out1,   // sigma (GAUSS)
                                                               int Hkv, int P, int Mmax, float scale,
                                                               int group_max, const ScoreAppend ap) {
  constexpr bool GAUSS = KIND == kKindGauss, BOX8 = KIND == kKindBox8;
  constexpr int TILE = score_tile(KIND), NT = TILE / 16;   // NT groups of 4 pages per wavefront
  constexpr int NSET = (G + 3) / 4;                 // column sets of 4 heads
  __shared__ float stage[2][G][TILE];
  const TileWork tw = score_work<bf16_t, APPEND>(ap, seq_lens, Hkv, P, Mmax, TILE);
  if (!tw.run) return;                               // workgroup-uniform
  const int b = tw.b, h = tw.h, tile0 = tw.tile0;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int m = lane & 15, j = lane >> 4;           // MFMA row / column index, K group
  const int pg = m >> 2, kq = m & 3;                // as a row: page of the group, channel quarter
  const int n = tw.n;
  const int M = (n + P - 1) / P;
  const int Hq = Hkv * G;
  if (tile0 >= M) {                                  // tile past the end of the sequence: no statistics are read
    for (int idx = threadIdx.x; idx < (group_max ? 1 : G) * TILE; idx += 256) {
      const int g = idx / TILE, p = tile0 + idx - g * TILE;
      if (p >= Mmax) continue;
      const size_t o = group_max ? ((size_t)b * Hkv + h) * Mmax + p : ((size_t)b * Hq + h * G + g) * Mmax + p;
      out0[o] = -INFINITY;
      if (GAUSS) out1[o] = 0.f;
    }
    return;
  }

  // B operands: column (g = m>>2, quarter kq) holds q[g][kq*32 + j*8 .. +8] (zero for g >= G)
  uint4 b0[NSET], b1[NSET], b2[NSET];
#pragma unroll
  for (int s = 0; s < NSET; ++s) {
    const int g = 4 * s + (m >> 2);
    uint4 qv = make_uint4(0, 0, 0, 0);
    if (g < G) qv = *reinterpret_cast<const uint4*>(q + ((size_t)b * Hq + h * G + g) * kD + kq * 32 + j * 8);
    if (GAUSS) {
      b0[s] = qv;
      square_split(qv.x, b1[s].x, b2[s].x); square_split(qv.y, b1[s].y, b2[s].y);
      square_split(qv.z, b1[s].z, b2[s].z); square_split(qv.w, b1[s].w, b2[s].w);
    } else {
      b0[s] = make_uint4(keep_sign<true>(qv.x), keep_sign<true>(qv.y), keep_sign<true>(qv.z), keep_sign<true>(qv.w));
      b1[s] = make_uint4(keep_sign<false>(qv.x), keep_sign<false>(qv.y), keep_sign<false>(qv.z), keep_sign<false>(qv.w));
      b2[s] = make_uint4(0, 0, 0, 0);
    }
  }

  const int pw0 = tile0 + w * (TILE / 4);            // first page of this wavefront
  uint4 a[BOX8 ? 1 : NT][2];
  uint4 raw[BOX8 ? NT : 1];
  if constexpr (BOX8) {
    // one 16-byte unit per lane and page: k_min and k_max codes of the lane's 8 channels
    const uint8_t* base8 = (const uint8_t*)stats_any + (((size_t)b * Hkv + h) * Mmax) * 256 + (kq * 4 + j) * 16;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int p = min(pw0 + 4 * t + pg, M - 1);   // clamped: pages past the end are masked on output
      raw[t] = *reinterpret_cast<const uint4*>(base8 + (size_t)p * 256);
    }
  } else {
    const bf16_t* base = (const bf16_t*)stats_any + (((size_t)b * Hkv + h) * Mmax) * 2 * kD + (kq * 4 + j) * 8;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const int p = min(pw0 + 4 * t + pg, M - 1);   // clamped: pages past the end are masked on output
#pragma unroll
      for (int s = 0; s < 2; ++s) a[t][s] = *reinterpret_cast<const uint4*>(base + ((size_t)p * 2 + s) * kD);
    }
  }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const int pt = w * (TILE / 4) + 4 * t + j;       // result row group j = page of the group
    const int ta = BOX8 ? 0 : t;
    if constexpr (BOX8) {                            // codes -> bf16 just before use (exact)
      a[0][0] = e4m3x8_to_bf16x8(raw[t].x, raw[t].y);
      a[0][1] = e4m3x8_to_bf16x8(raw[t].z, raw[t].w);
    }
#pragma unroll
    for (int s = 0; s < NSET; ++s) {
      const int g = 4 * s + (m >> 2);
      const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
      if (GAUSS) {
        const f32x4_t c0 = mfma_bf16(a[ta][0], b0[s], zero);
        f32x4_t c1 = mfma_bf16(a[ta][1], b1[s], zero);
        c1 = mfma_bf16(a[ta][1], b2[s], c1);
        const float mu = diag_quad_sum(c0, kq), var = diag_quad_sum(c1, kq);
        if (kq == 0 && g < G) { stage[0][g][pt] = scale * mu; stage[1][g][pt] = scale * sqrtf(fmaxf(var, 0.f)); }
      } else {
        f32x4_t c0 = mfma_bf16(a[ta][0], b0[s], zero);
        c0 = mfma_bf16(a[ta][1], b1[s], c0);
        const float v = diag_quad_sum(c0, kq);
        // a bound the 8-bit format could not hold is NaN: such a page scores +inf (always selected)
        if (kq == 0 && g < G) stage[0][g][pt] = (BOX8 && v != v) ? INFINITY : scale * v;
      }
    }
  }
  __syncthreads();
  if (group_max) {                                   // one score per page and KV head: the group's maximum
    for (int pt = threadIdx.x; pt < TILE; pt += 256) {
      const int p = tile0 + pt;
      if (p >= Mmax) continue;
      float v = stage[0][0][pt];
#pragma unroll
      for (int g = 1; g < G; ++g) v = fmaxf(v, stage[0][g][pt]);
      out0[((size_t)b * Hkv + h) * Mmax + p] = p < M ? v : -INFINITY;
    }
    return;
  }
  for (int idx = threadIdx.x; idx < G * TILE; idx += 256) {
    const int g = idx / TILE, pt = idx - g * TILE;
    const int p = tile0 + pt;
    if (p >= Mmax) continue;
    const size_t o = ((size_t)b * Hq + h * G + g) * Mmax + p;
    const bool valid = p < M;
    out0[o] = valid ? stage[0][g][pt] : -INFINITY;
    if (GAUSS) out1[o] = valid ? stage[1][g][pt] : 0.f;
  }
}

// float32 statistics: one wavefront step = two page records, 32 lanes x 8 channels each.
template <int G, bool GAUSS, bool APPEND>
__global__ __launch_bounds__(256) void score_pages_f32_kernel(const float* __restrict__ q,
                                                              const float* __restrict__ stats,
                                                              const int32_t* __restrict__ seq_lens,
                                                              float* __restrict__ out0, float* __restrict__ out1,
                                                              int Hkv, int P, int Mmax, float scale, int group_max,
                                                              const ScoreAppend ap) {
  constexpr int kSteps = kScoreTile / 4 / 2;
  __shared__ float stage[2][G][kScoreTile];
  const TileWork tw = score_work<float, APPEND>(ap, seq_lens, Hkv, P, Mmax, kScoreTile);
  if (!tw.run) return;                               // workgroup-uniform
  const int b = tw.b, h = tw.h, tile0 = tw.tile0;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int half = lane >> 5, which = (lane >> 4) & 1, c = lane & 15;
  const int n = tw.n;
  const int M = (n + P - 1) / P;
  const int Hq = Hkv * G;
  if (tile0 >= M) {                                  // tile past the end of the sequence: no statistics are read
    for (int idx = threadIdx.x; idx < (group_max ? 1 : G) * kScoreTile; idx += 256) {
      const int g = idx / kScoreTile, p = tile0 + idx - g * kScoreTile;
      if (p >= Mmax) continue;
      const size_t o = group_max ? ((size_t)b * Hkv + h) * Mmax + p : ((size_t)b * Hq + h * G + g) * Mmax + p;
      out0[o] = -INFINITY;
      if (GAUSS) out1[o] = 0.f;
    }
    return;
  }
  float coef[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float qv[8];
    load8<float>(q + ((size_t)b * Hq + h * G + g) * kD + 8 * c, qv);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (GAUSS) coef[g][i] = which ? qv[i] * qv[i] : qv[i];
      else       coef[g][i] = which ? fmaxf(qv[i], 0.f) : fminf(qv[i], 0.f);
    }
  }
  const int pw0 = tile0 + w * (kScoreTile / 4);
  const float* base = stats + (((size_t)b * Hkv + h) * Mmax) * 2 * kD;
  for (int it = 0; it < kSteps; ++it) {
    const int p = min(pw0 + 2 * it + half, M - 1);  // clamped: pages past the end are masked on output
    const int pt = w * (kScoreTile / 4) + 2 * it + half;
    float x[8];
    load8<float>(base + ((size_t)p * 2 + which) * kD + 8 * c, x);
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc = fmaf(coef[g][i], x[i], acc);
      acc = row16_sum(acc);
      if (GAUSS) {
        if (c == 0) stage[which][g][pt] = which ? scale * sqrtf(fmaxf(acc, 0.f)) : scale * acc;
      } else {
        acc += __shfl_xor(acc, 16);
        if (c == 0 && which == 0) stage[0][g][pt] = scale * acc;
      }
    }
  }
  __syncthreads();
  if (group_max) {                                   // one score per page and KV head: the group's maximum
    for (int pt = threadIdx.x; pt < kScoreTile; pt += 256) {
      const int p = tile0 + pt;
      if (p >= Mmax) continue;
      float v = stage[0][0][pt];
#pragma unroll
      for (int g = 1; g < G; ++g) v = fmaxf(v, stage[0][g][pt]);
      out0[((size_t)b * Hkv + h) * Mmax + p] = p < M ? v : -INFINITY;
    }
    return;
  }
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

// One-dimensional grid over (unit, tile) plus the appending workgroups, folded over x and y.
static dim3 score_grid(const Dims& dm, int tile, bool appending, ScoreAppend* ap) {
  ap->units = dm.Hkv * dm.B;
  ap->n_tiles = (dm.Mmax + tile - 1) / tile;
  const long long total = (long long)ap->units * ap->n_tiles + (appending ? ap->units : 0);
  const long long gx = total < (1 << 20) ? total : (1 << 20);
  return dim3((unsigned)gx, (unsigned)((total + gx - 1) / gx));
}

template <int G, bool APPEND>
static void launch_score_GA(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                           int mode, float* box, float* mu, float* sigma, hipStream_t st, const ScoreAppend& ap0) {
  dim3 block(256);
  const int gmax = (mode & EKV_SCORE_GROUP_MAX) ? 1 : 0;
  // with both score kinds requested the first launch appends, the second only scores with the new length
  ScoreAppend ap_box = ap0, ap_gauss = ap0;
  if (ap0.mode == 1 && (mode & EKV_SCORE_BOX)) ap_gauss.mode = 2;
  const dim3 grid = score_grid(dm, kScoreTile, APPEND && ap_box.mode == 1, &ap_box);       // 512-byte records
  const dim3 grid_g = score_grid(dm, kScoreTile, APPEND && ap_gauss.mode == 1, &ap_gauss);
  if (dm.dtype == EKV_BF16) {
    if (mode & EKV_SCORE_BOX8) {
      ScoreAppend ap8 = ap_box;
      const dim3 grid8 = score_grid(dm, score_tile(kKindBox8), APPEND && ap8.mode == 1, &ap8);
      hipLaunchKernelGGL((score_pages_mfma_kernel<G, kKindBox8, APPEND>), grid8, block, 0, st, (const bf16_t*)q,
                         (const void*)s.box8, seq_lens, box, (float*)nullptr, dm.Hkv, dm.P, dm.Mmax, dm.scale, gmax, ap8);
    }
    if (mode & EKV_SCORE_BOX)
      hipLaunchKernelGGL((score_pages_mfma_kernel<G, kKindBox, APPEND>), grid, block, 0, st, (const bf16_t*)q,
                         (const void*)s.box, seq_lens, box, (float*)nullptr, dm.Hkv, dm.P, dm.Mmax, dm.scale, gmax, ap_box);
    if (mode & EKV_SCORE_GAUSS)
      hipLaunchKernelGGL((score_pages_mfma_kernel<G, kKindGauss, APPEND>), grid_g, block, 0, st, (const bf16_t*)q,
                         (const void*)s.gauss, seq_lens, mu, sigma, dm.Hkv, dm.P, dm.Mmax, dm.scale, 0, ap_gauss);
  } else {
    if (mode & EKV_SCORE_BOX)
      hipLaunchKernelGGL((score_pages_f32_kernel<G, false, APPEND>), grid, block, 0, st, (const float*)q,
                         (const float*)s.box, seq_lens, box, (float*)nullptr, dm.Hkv, dm.P, dm.Mmax, dm.scale, gmax, ap_box);
    if (mode & EKV_SCORE_GAUSS)
      hipLaunchKernelGGL((score_pages_f32_kernel<G, true, APPEND>), grid_g, block, 0, st, (const float*)q,
                         (const float*)s.gauss, seq_lens, mu, sigma, dm.Hkv, dm.P, dm.Mmax, dm.scale, 0, ap_gauss);
  }
}

template <int G>
static void launch_score_G(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                           int mode, float* box, float* mu, float* sigma, hipStream_t st, const ScoreAppend& ap) {
  if (ap.mode == 1) launch_score_GA<G, true>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap);
  else launch_score_GA<G, false>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap);
}

void launch_score_pages(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                        int mode, float* box, float* mu, float* sigma, hipStream_t st, const ekv_cache_view* append_to,
                        const void* k_new, const void* v_new) {
  ScoreAppend ap{nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, 0, 0, dm.HkvPool, 0, 0};
  if (append_to != nullptr) {
    ap = ScoreAppend{append_to->k_pool, append_to->v_pool, append_to->block_table, k_new, v_new, s.box, s.gauss,
                     s.box8, append_to->n_phys_pages, 1, dm.HkvPool, 0, 0};
    if (dm.P > 32) {
      // Inside the scoring launch a page other than 16 tokens is read row by row (a batch of loads per lane
      // would raise the register count of the kernel, which sets the occupancy of the whole stream): 16
      // dependent loads for 64 tokens, and the launch is as long as that chain (23 us instead of 14 at 8192
      // pages).  Such pages take the append kernel first (one batch of loads there); the scoring launch then
      // only counts the new token (mode 2).  Up to 32 tokens the chain is short enough to stay inside.
      launch_stats_append(dm, *append_to, s, k_new, v_new, st);
      ap.mode = 2;
    }
  }
  switch (dm.G) {
    case 1: launch_score_G<1>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap); break;
    case 2: launch_score_G<2>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap); break;
    case 4: launch_score_G<4>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap); break;
    default: launch_score_G<8>(dm, q, s, seq_lens, mode, box, mu, sigma, st, ap); break;
  }
}

}  // namespace ekv
