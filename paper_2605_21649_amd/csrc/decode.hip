// Sparse and dense alpha-entmax decode (paper Sec. 4.1, Sec. 4.4; Eq. 1-3).
//
// Entmax has no online rescaling: the threshold tau needs every candidate score.  The work is split:
//   pass 1 (many workgroups, HBM-bound): gather the K pages, z_j = a*scale*q.k_j, write z (4 B/token)
//           and one maximum per chunk of pages to scratch.
//   pass 2 (one workgroup per (b,h)): zmax from the chunk maxima; only z > zmax-1 can be in the
//           support (at tau = zmax-1 the largest entry alone has mass 1), and chunks whose maximum is
//           below that are skipped; the survivors are compacted IN ORDER into LDS; tau is solved
//           there; p_j = (z_j - tau)^beta; V rows are gathered only where p_j > 0.
// All reductions have a fixed order, so results are bit-reproducible.
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kScoreThreads = 256;
constexpr int kSolveThreads = 1024;
constexpr int kSolveWaves = kSolveThreads / 64;
constexpr int kListCap = 6144;          // candidate entries held in LDS (u, pos): 48 KB

// ------------------------------------------------------------------------------------------
// pass 1: scores
// ------------------------------------------------------------------------------------------
// DENSE: unit = (b, KV head); the G query heads of the group are scored from one read of K.
// sparse: unit = (b, query head) with its own page list (G = 1).
template <typename T, int G, bool DENSE, int PT>   // PT = compile-time page size, 0 = runtime
__global__ __launch_bounds__(kScoreThreads) void decode_scores_kernel(
    const T* __restrict__ q, const T* __restrict__ k_pool, const int32_t* __restrict__ block_table,
    const int32_t* __restrict__ seq_lens, const int32_t* __restrict__ page_idx,
    const int32_t* __restrict__ n_sel, float* __restrict__ zbuf, float* __restrict__ pmax, int Hq, int Hkv,
    int P_rt, int Mmax, int cap, size_t zstride, int n_chunks_max, float zscale) {
  __shared__ float wmax_s[kScoreThreads / 64][G];
  const int P = PT ? PT : P_rt;
  const int unit = blockIdx.y, chunk = blockIdx.x;
  const int b = DENSE ? unit / Hkv : unit / Hq;
  const int hkv = DENSE ? unit % Hkv : (unit % Hq) / (Hq / Hkv);
  const int hq0 = DENSE ? hkv * G : unit % Hq;            // first (only) query head of this unit
  const int n = seq_lens[b];
  const int n_slots = DENSE ? (n + P - 1) / P : n_sel[unit];
  const int slot0 = chunk * kPagesPerScoreBlock;
  if (slot0 >= n_slots) return;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = lane >> 4, c = lane & 15;

  float coef[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) load8<T>(q + ((size_t)b * Hq + hq0 + g) * kD + 8 * c, coef[g]);

  float wmax[G];
#pragma unroll
  for (int g = 0; g < G; ++g) wmax[g] = -INFINITY;

  constexpr int kPagesPerWave = kPagesPerScoreBlock / (kScoreThreads / 64);
#pragma unroll
  for (int pw = 0; pw < kPagesPerWave; ++pw) {
    const int slot = slot0 + w * kPagesPerWave + pw;
    if (slot >= n_slots) break;
    const int lp = DENSE ? slot : page_idx[(size_t)unit * cap + slot];
    const int phys = block_table[(size_t)b * Mmax + lp];
    const T* kpage = k_pool + ((size_t)phys * Hkv + hkv) * P * kD + 8 * c;
    float zkeep[G];
#pragma unroll
    for (int g = 0; g < G; ++g) zkeep[g] = -INFINITY;
    if constexpr (PT != 0) {
      float x[PT ? PT / 4 : 1][8];
#pragma unroll
      for (int s = 0; s < PT / 4; ++s) load8<T>(kpage + (size_t)(4 * s + r) * kD, x[s]);
#pragma unroll
      for (int s = 0; s < PT / 4; ++s) {
        const bool valid = lp * P + 4 * s + r < n;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float acc = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc = fmaf(coef[g][i], x[s][i], acc);
          acc = row16_sum(acc);
          const float z = valid ? zscale * acc : -INFINITY;
          if (c == s) zkeep[g] = z;
          wmax[g] = fmaxf(wmax[g], z);
        }
      }
    } else {
      for (int s = 0; s < P / 4; ++s) {
        float x[8];
        load8<T>(kpage + (size_t)(4 * s + r) * kD, x);
        const bool valid = lp * P + 4 * s + r < n;
#pragma unroll
        for (int g = 0; g < G; ++g) {
          float acc = 0.f;
#pragma unroll
          for (int i = 0; i < 8; ++i) acc = fmaf(coef[g][i], x[i], acc);
          acc = row16_sum(acc);
          const float z = valid ? zscale * acc : -INFINITY;
          if (c == s) zkeep[g] = z;
          wmax[g] = fmaxf(wmax[g], z);
        }
      }
    }
    if (c < P / 4) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const size_t row = DENSE ? (size_t)b * Hq + hq0 + g : (size_t)unit;
        zbuf[row * zstride + (size_t)slot * P + 4 * c + r] = zkeep[g];
      }
    }
  }
#pragma unroll
  for (int g = 0; g < G; ++g) {
    float m = wmax[g];
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    if (lane == 0) wmax_s[w][g] = m;
  }
  __syncthreads();
  if (threadIdx.x < G) {
    const int g = threadIdx.x;
    float m = wmax_s[0][g];
    for (int i = 1; i < kScoreThreads / 64; ++i) m = fmaxf(m, wmax_s[i][g]);
    const size_t row = DENSE ? (size_t)b * Hq + hq0 + g : (size_t)unit;
    pmax[row * n_chunks_max + chunk] = m;
  }
}

// ------------------------------------------------------------------------------------------
// pass 2: threshold, probabilities, weighted value sum
// ------------------------------------------------------------------------------------------
struct SolveShared {
  float list_u[kListCap];         // z - zmax of the candidates that can be in the support
  int32_t list_pos[kListCap];     // their position in the candidate order
  float obuf[kSolveWaves][kD];
  float red[2][kSolveWaves][3];
  int wcount[kSolveWaves];
  float red1[kSolveWaves];
};

// Candidate source: the compacted LDS list, or (when it does not fit) the score row itself.
struct ListSrc {
  const float* u; const int32_t* pos; int n;
  __device__ __forceinline__ float get_u(int i) const { return u[i]; }
  __device__ __forceinline__ int get_pos(int i) const { return pos[i]; }
};
struct RowSrc {
  const float* z; int n; float zmax;
  __device__ __forceinline__ float get_u(int i) const { return z[i] - zmax; }
  __device__ __forceinline__ int get_pos(int i) const { return i; }
};

// F = sum (u-tau)_+^beta, D = beta * sum (u-tau)_+^(beta-1), cnt = #{u > tau}; one barrier per call
// (double-buffered by `parity`).
template <typename Src>
__device__ __forceinline__ void eval_mass(const Src& src, float tau, float beta, int ibeta, SolveShared& sh,
                                          int parity, float& F, float& D, int& cnt) {
  float f = 0.f, d = 0.f; int c = 0;
  for (int i = threadIdx.x; i < src.n; i += kSolveThreads) {
    const float x = src.get_u(i) - tau;
    if (x > 0.f) { f += pow_beta(x, beta, ibeta); d += pow_beta_m1(x, beta, ibeta); ++c; }
  }
  f = wave_sum(f); d = wave_sum(d); c = wave_sum_i(c);
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sh.red[parity][w][0] = f; sh.red[parity][w][1] = d; sh.red[parity][w][2] = __int_as_float(c); }
  __syncthreads();
  float Fs = 0.f, Ds = 0.f; int Cs = 0;
  for (int i = 0; i < kSolveWaves; ++i) {
    Fs += sh.red[parity][i][0]; Ds += sh.red[parity][i][1]; Cs += __float_as_int(sh.red[parity][i][2]);
  }
  F = Fs; D = beta * Ds; cnt = Cs;
}

// Root of sum (u - tau)_+^beta = 1 for u <= 0 with max u = 0: tau in [-1, 0).
// Safeguarded iteration inside a bracket [lo,hi], F(lo) >= 1 > F(hi).  From a left point the step is
// the exact root for the current support when beta is 1 or 2 (closed forms), Newton otherwise; from a
// right point a Newton step (F is convex, so it lands left of the root).  For beta in {1,2} the root is
// accepted as exact once a closed-form step leaves the support count unchanged.
template <typename Src>
__device__ __forceinline__ float solve_tau(const Src& src, float beta, int ibeta, SolveShared& sh, int& supp) {
  float lo = -1.0f - 4e-6f, hi = 0.f;
  float tau = lo;
  int pending_cnt = -1;
  int parity = 0, cnt = 0;
  for (int it = 0; it < 64; ++it) {
    float F, D;
    eval_mass(src, tau, beta, ibeta, sh, parity, F, D, cnt);
    parity ^= 1;
    if (pending_cnt >= 0 && cnt == pending_cnt) break;       // exact step kept the support: done
    pending_cnt = -1;
    float step;
    if (F >= 1.0f) {
      lo = tau;
      const float e = F - 1.0f;
      if (ibeta == 1) { step = e / (float)cnt; pending_cnt = cnt; }
      else if (ibeta == 2) {
        const float A = 0.5f * D;                            // sum (u - tau)
        const float disc = fmaf(A, A, -(float)cnt * e);
        if (disc > 0.f) { step = e / (A + sqrtf(disc)); pending_cnt = cnt; }
        else step = e / D;
      } else step = e / D;
    } else {
      hi = tau;
      step = D > 0.f ? (F - 1.0f) / D : -INFINITY;
    }
    float next = tau + step;
    if (!(next > lo && next < hi)) { next = 0.5f * (lo + hi); pending_cnt = -1; }
    if (next == tau || hi - lo <= 1.2e-7f) { tau = next; pending_cnt = -2; break; }
    if (pending_cnt < 0 && fabsf(next - tau) <= 1.2e-7f) { tau = next; pending_cnt = -2; break; }
    tau = next;
  }
  if (pending_cnt == -2) {                                     // tau moved after the last evaluation
    float F, D;
    eval_mass(src, tau, beta, ibeta, sh, parity, F, D, cnt);
  }
  supp = cnt;
  return tau;
}

template <typename T, bool DENSE>
__device__ __forceinline__ const T* v_row_ptr(const T* v_pool, const int32_t* block_table,
                                              const int32_t* page_idx, int b, int bh, int hkv, int Hkv, int P,
                                              int Mmax, int cap, int pos) {
  const int slot = pos / P, tok = pos - slot * P;
  const int lp = DENSE ? slot : page_idx[(size_t)bh * cap + slot];
  const int phys = block_table[(size_t)b * Mmax + lp];
  return v_pool + (((size_t)phys * Hkv + hkv) * P + tok) * kD;
}

template <typename T, bool DENSE, typename Src>
__device__ __forceinline__ void weighted_values(const Src& src, float tau, float beta, int ibeta,
                                                const T* __restrict__ v_pool,
                                                const int32_t* __restrict__ block_table,
                                                const int32_t* __restrict__ page_idx, int b, int bh, int hkv,
                                                int Hkv, int P, int Mmax, int cap, SolveShared& sh,
                                                float* __restrict__ out) {
  const int tid = threadIdx.x, rs = tid >> 4, c = tid & 15, w = tid >> 6;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  for (int e = rs; e < src.n; e += kSolveThreads / 16) {
    const float x = src.get_u(e) - tau;
    if (x > 0.f) {
      const float p = pow_beta(x, beta, ibeta);
      float v[8];
      load8<T>(v_row_ptr<T, DENSE>(v_pool, block_table, page_idx, b, bh, hkv, Hkv, P, Mmax, cap, src.get_pos(e)) + 8 * c, v);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = fmaf(p, v[i], acc[i]);
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc[i] += __shfl_xor(acc[i], 16);
    acc[i] += __shfl_xor(acc[i], 32);
  }
  __syncthreads();
  if ((tid & 63) < 16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) sh.obuf[w][8 * c + i] = acc[i];
  }
  __syncthreads();
  if (tid < kD) {
    float s = 0.f;
    for (int i = 0; i < kSolveWaves; ++i) s += sh.obuf[i][tid];
    out[(size_t)bh * kD + tid] = s;
  }
}

// Ordered list of the support's logical token indices (side output).
template <bool DENSE, typename Src>
__device__ __forceinline__ void write_support(const Src& src, float tau, const int32_t* __restrict__ page_idx,
                                              int bh, int P, int cap, SolveShared& sh,
                                              int32_t* __restrict__ dst, int dst_cap) {
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  int base = 0;
  for (int i0 = 0; i0 < src.n; i0 += kSolveThreads) {
    const int i = i0 + tid;
    const bool in = i < src.n && src.get_u(i) > tau;
    const uint64_t m = __ballot(in);
    __syncthreads();
    if (lane == 0) sh.wcount[w] = __popcll(m);
    __syncthreads();
    int off = base, tot = 0;
    for (int j = 0; j < kSolveWaves; ++j) { const int cj = sh.wcount[j]; if (j < w) off += cj; tot += cj; }
    if (in) {
      off += __popcll(m & ((1ull << lane) - 1ull));
      if (off < dst_cap) {
        const int pos = src.get_pos(i);
        const int slot = pos / P, tok = pos - slot * P;
        const int lp = DENSE ? slot : page_idx[(size_t)bh * cap + slot];
        dst[off] = lp * P + tok;
      }
    }
    base += tot;
  }
}

template <typename T, bool DENSE>
__global__ __launch_bounds__(kSolveThreads) void decode_solve_kernel(
    const T* __restrict__ v_pool, const int32_t* __restrict__ block_table, const int32_t* __restrict__ seq_lens,
    const int32_t* __restrict__ page_idx, const int32_t* __restrict__ n_sel, const float* __restrict__ zbuf,
    const float* __restrict__ pmax, float* __restrict__ out, float* __restrict__ tau_out,
    int32_t* __restrict__ supp_out, ekv_decode_extras ex, int Hq, int Hkv, int P, int Mmax, int cap,
    size_t zstride, int n_chunks_max, float a, float beta, int ibeta) {
  __shared__ SolveShared sh;
  const int bh = blockIdx.x, b = bh / Hq, hq = bh % Hq, hkv = hq / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int n = seq_lens[b];
  const int n_slots = DENSE ? (n + P - 1) / P : n_sel[bh];
  const int n_cand = n_slots * P;
  const int n_chunks = (n_slots + kPagesPerScoreBlock - 1) / kPagesPerScoreBlock;
  const int chunk_tokens = kPagesPerScoreBlock * P;
  const float* zr = zbuf + (size_t)bh * zstride;
  const float* pm = pmax + (size_t)bh * n_chunks_max;

  float m = -INFINITY;
  for (int i = tid; i < n_chunks; i += kSolveThreads) m = fmaxf(m, pm[i]);
  const float zmax = block_max(m, sh.red1);
  if (!(zmax > -INFINITY)) {                // no valid candidate at all
    if (tid < kD) out[(size_t)bh * kD + tid] = 0.f;
    if (tid == 0) { tau_out[bh] = INFINITY; supp_out[bh] = 0; }
    return;
  }
  const float thr = zmax - 1.0f - 4e-6f * fmaxf(1.f, fabsf(zmax));

  // ordered compaction of {z > thr}: wavefront w owns a contiguous range of chunks
  const int cpw = (n_chunks + kSolveWaves - 1) / kSolveWaves;
  const int ck0 = min(w * cpw, n_chunks), ck1 = min(ck0 + cpw, n_chunks);
  int wc = 0;
  for (int ck = ck0; ck < ck1; ++ck) {
    if (!(pm[ck] > thr)) continue;
    const int base = ck * chunk_tokens;
    for (int j = lane; j < chunk_tokens; j += 64) {
      const int pos = base + j;
      const bool in = pos < n_cand && zr[pos] > thr;
      wc += __popcll(__ballot(in));
    }
  }
  __syncthreads();
  if (lane == 0) sh.wcount[w] = wc;
  __syncthreads();
  int woff = 0, n_list = 0;
  for (int j = 0; j < kSolveWaves; ++j) { const int cj = sh.wcount[j]; if (j < w) woff += cj; n_list += cj; }
  const bool in_lds = n_list <= kListCap;
  if (in_lds) {
    for (int ck = ck0; ck < ck1; ++ck) {
      if (!(pm[ck] > thr)) continue;
      const int base = ck * chunk_tokens;
      for (int j = lane; j < chunk_tokens; j += 64) {
        const int pos = base + j;
        const float z = pos < n_cand ? zr[pos] : -INFINITY;
        const bool in = z > thr;
        const uint64_t mk = __ballot(in);
        if (in) {
          const int o = woff + __popcll(mk & ((1ull << lane) - 1ull));
          sh.list_u[o] = z - zmax;
          sh.list_pos[o] = pos;
        }
        woff += __popcll(mk);
      }
    }
  }
  __syncthreads();

  float tau_u; int supp;
  const ListSrc ls{sh.list_u, sh.list_pos, n_list};
  const RowSrc rs{zr, n_cand, zmax};
  if (in_lds) {
    tau_u = solve_tau(ls, beta, ibeta, sh, supp);
    weighted_values<T, DENSE>(ls, tau_u, beta, ibeta, v_pool, block_table, page_idx, b, bh, hkv, Hkv, P, Mmax, cap, sh, out);
  } else {
    tau_u = solve_tau(rs, beta, ibeta, sh, supp);
    weighted_values<T, DENSE>(rs, tau_u, beta, ibeta, v_pool, block_table, page_idx, b, bh, hkv, Hkv, P, Mmax, cap, sh, out);
  }
  const float tau = tau_u + zmax;
  if (tid == 0) { tau_out[bh] = tau; supp_out[bh] = supp; }

  // ---- optional side outputs ------------------------------------------------------------
  if (ex.support_tokens != nullptr) {
    int32_t* dst = ex.support_tokens + (size_t)bh * ex.support_cap;
    if (in_lds) write_support<DENSE>(ls, tau_u, page_idx, bh, P, cap, sh, dst, ex.support_cap);
    else write_support<DENSE>(rs, tau_u, page_idx, bh, P, cap, sh, dst, ex.support_cap);
  }
  if (ex.tau_ref != nullptr && (ex.kept_mass_ref != nullptr || ex.kept_supp_ref != nullptr)) {
    const float tr = ex.tau_ref[bh];
    float f = 0.f; int c = 0;
    for (int i = tid; i < n_cand; i += kSolveThreads) {
      const float x = zr[i] - tr;
      if (x > 0.f) { f += pow_beta(x, beta, ibeta); ++c; }
    }
    f = block_sum(f, sh.red1);
    c = block_sum_i(c, sh.wcount);
    if (tid == 0) {
      if (ex.kept_mass_ref != nullptr) ex.kept_mass_ref[bh] = f;
      if (ex.kept_supp_ref != nullptr) ex.kept_supp_ref[bh] = c;
    }
  }
  if (DENSE && ex.lse != nullptr) {
    // log sum_j exp(s_j) with s_j = z_j / a, shifted by the maximum
    const float inv_a = 1.0f / a;
    float f = 0.f;
    for (int i = tid; i < n_cand; i += kSolveThreads) f += __expf((zr[i] - zmax) * inv_a);
    f = block_sum(f, sh.red1);
    if (tid == 0) ex.lse[bh] = zmax * inv_a + __logf(f);
  }
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
template <typename T, int G, bool DENSE>
static void launch_scores_P(const Dims& dm, dim3 grid, const void* q, const ekv_cache_view& c,
                            const int32_t* page_idx, const int32_t* n_sel, const DecodeWorkspace& ws,
                            hipStream_t st) {
  const float zscale = dm.a * dm.scale;
#define EKV_SCORES(PT)                                                                                        \
  hipLaunchKernelGGL((decode_scores_kernel<T, G, DENSE, PT>), grid, dim3(kScoreThreads), 0, st, (const T*)q,  \
                     (const T*)c.k_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws.z, ws.pmax, dm.Hq,    \
                     dm.Hkv, dm.P, dm.Mmax, dm.cap, ws.zstride, ws.n_chunks_max, zscale)
  if (dm.P == 16) EKV_SCORES(16);
  else if (dm.P == 32) EKV_SCORES(32);
  else EKV_SCORES(0);
#undef EKV_SCORES
}

template <typename T>
static void launch_decode_T(const Dims& dm, bool dense, const void* q, const ekv_cache_view& c,
                            const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                            int32_t* supp, const ekv_decode_extras& ex, const DecodeWorkspace& ws,
                            hipStream_t st) {
  if (dense) {
    dim3 grid(ws.n_chunks_max, dm.B * dm.Hkv);
    switch (dm.G) {
      case 1: launch_scores_P<T, 1, true>(dm, grid, q, c, page_idx, n_sel, ws, st); break;
      case 2: launch_scores_P<T, 2, true>(dm, grid, q, c, page_idx, n_sel, ws, st); break;
      case 4: launch_scores_P<T, 4, true>(dm, grid, q, c, page_idx, n_sel, ws, st); break;
      default: launch_scores_P<T, 8, true>(dm, grid, q, c, page_idx, n_sel, ws, st); break;
    }
    hipLaunchKernelGGL((decode_solve_kernel<T, true>), dim3(dm.B * dm.Hq), dim3(kSolveThreads), 0, st,
                       (const T*)c.v_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws.z, ws.pmax, out, tau,
                       supp, ex, dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, ws.zstride, ws.n_chunks_max, dm.a,
                       dm.beta, dm.ibeta);
  } else {
    dim3 grid(ws.n_chunks_max, dm.B * dm.Hq);
    launch_scores_P<T, 1, false>(dm, grid, q, c, page_idx, n_sel, ws, st);
    hipLaunchKernelGGL((decode_solve_kernel<T, false>), dim3(dm.B * dm.Hq), dim3(kSolveThreads), 0, st,
                       (const T*)c.v_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws.z, ws.pmax, out, tau,
                       supp, ex, dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, ws.zstride, ws.n_chunks_max, dm.a,
                       dm.beta, dm.ibeta);
  }
}

void launch_decode(const Dims& dm, bool dense, const void* q, const ekv_cache_view& c,
                   const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau, int32_t* supp,
                   const ekv_decode_extras& ex, const DecodeWorkspace& ws, hipStream_t st) {
  if (dm.dtype == EKV_F32) launch_decode_T<float>(dm, dense, q, c, page_idx, n_sel, out, tau, supp, ex, ws, st);
  else launch_decode_T<bf16_t>(dm, dense, q, c, page_idx, n_sel, out, tau, supp, ex, ws, st);
}

}  // namespace ekv
