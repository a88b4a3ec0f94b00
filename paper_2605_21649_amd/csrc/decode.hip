// Sparse and dense alpha-entmax decode (paper Sec. 4.1, Sec. 4.4; Eq. 1-3).
//
// Entmax has no online rescaling: the threshold tau needs every candidate score.  The work is split:
//   pass 1 (many workgroups, HBM-bound): gather the K pages, z_j = a*scale*q.k_j, write z (4 B/token)
//           and one maximum per group of pages (64 tokens) to scratch.  bf16 pages go through the matrix cores:
//           an MFMA tile's 16 rows are 4 tokens x 4 channel quarters, so each lane's A operand is the
//           16 bytes of a fully coalesced load, its 16 columns are (query head, channel quarter); the
//           blocks with matching quarters are summed with two DPP quad steps.
//   pass 2 (one workgroup per (b,h)): zmax from the chunk maxima; only z > zmax-1 can be in the
//           support (at tau = zmax-1 the largest entry alone has mass 1), and chunks whose maximum is
//           below that are not read; the survivors are compacted IN ORDER into LDS; tau is solved
//           there; p_j = (z_j - tau)^beta; V rows are gathered only where p_j > 0.
// All reductions have a fixed order, so results are bit-reproducible.
#include "ekv_device.h"
#include "ekv_internal.h"

namespace ekv {

constexpr int kScoreThreads = 256;
constexpr int kSolveThreads = 1024;
constexpr int kSolveWaves = kSolveThreads / 64;
constexpr int kListCap = 4096;          // candidate entries held in LDS (u, pos, row): 48 KB
constexpr int kSpillCap = 65536;        // entries of a row's overflow list in the workspace (longer lists: the row is streamed)
constexpr int kPreR = kPreGroups / kSolveThreads;    // group maxima a thread of the solve holds at most
constexpr int kRoundLoads = 16;         // loads per lane and compaction round
constexpr int kRoundTokens = kSolveThreads * kRoundLoads;

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

// ------------------------------------------------------------------------------------------
// pass 1: scores
// ------------------------------------------------------------------------------------------
// Candidate source of a launch: per query head its own page list (unit = (b, query head), G = 1);
// every page of the sequence; or one page list per KV head shared by its G query heads.  In the last
// two the unit is (b, KV head) and the G heads are scored from one read of K.
enum : int { kPerHead = 0, kAllPages = 1, kGroupList = 2 };

struct ScoreArgs {
  const void* q; const void* k_pool;
  const int32_t* block_table; const int32_t* seq_lens; const int32_t* page_idx; const int32_t* n_sel;
  float* zbuf; float* pmax;
  int Hq, Hkv, P, Mmax, cap, n_chunks_max, n_phys;
  size_t zstride;
  float zscale;
  int HkvPool;
  int U;                  // units of the launch: B*Hq page lists, or B*Hkv (all pages / one list per KV head)
  const int32_t* pre_g;   // exclusive prefix of the items per unit, [U + 1], when U is too large for LDS
};

constexpr int kScoreWaves = kScoreThreads / 64;
constexpr int kUnitsLdsMax = 8192;      // units whose item prefix a workgroup keeps in LDS (32 KB)

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return min(max(x, lo), hi); }
__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

// Work distribution of pass 1.  An item is one group of pmax_pages(P) page slots of one unit (64 tokens when P
// divides 64): the granularity of pmax.  The launch has a fixed number of wavefronts that does not depend on the
// capacity of the page lists: the items of all units, in (unit, group) order, form one sequence of T items, and
// wavefront i of W takes the contiguous range [i*T/W, (i+1)*T/W).  T and the unit boundaries come from the
// device-side lengths (n_sel, or seq_lens when every page is a candidate): every workgroup builds the exclusive
// prefix of the items per unit in LDS (launches with more units than LDS holds read it from `pre_g`, written by
// unit_prefix_kernel before).
template <int MODE>
__device__ __forceinline__ int unit_slots(const ScoreArgs& A, int u) {
  if (MODE == kAllPages) return clampi((A.seq_lens[u / A.Hkv] + A.P - 1) / A.P, 0, A.Mmax);
  return clampi(A.n_sel[u], 0, A.cap);
}

template <int MODE>
__global__ __launch_bounds__(1024) void unit_prefix_kernel(const ScoreArgs A, int32_t* pre_out) {
  __shared__ int wsum[16];
  const int gp = pmax_pages(A.P);
  block_exclusive_prefix<1024>(A.U, [&](int u) { return (unit_slots<MODE>(A, u) + gp - 1) / gp; }, pre_out, wsum);
}

// The item range of this wavefront and the unit its first item lies in.
struct WaveItems { int begin, end, unit; };
template <typename P>
__device__ __forceinline__ WaveItems wave_item_range(const P pre, int U, int w) {
  const int total = uniform(pre[U]);
  const int W = gridDim.x * kScoreWaves, gw = blockIdx.x * kScoreWaves + w;
  // balanced contiguous partition: the first total % W wavefronts take one item more
  const int per = total / W, rem = total - per * W;
  WaveItems r;
  r.begin = gw * per + min(gw, rem);
  r.end = r.begin + per + (gw < rem ? 1 : 0);
  int lo = 0, hi = U;                                   // pre[lo] <= begin < pre[hi] whenever begin < total
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (uniform(pre[mid]) <= r.begin) lo = mid; else hi = mid;
  }
  r.unit = lo;
  return r;
}

// Generic path (float32 caches, or page sizes that are not 16, 32 or 64): FMAs + DPP row sums.
template <typename T, int G, int MODE, bool PRE_GLOBAL>
__global__ __launch_bounds__(kScoreThreads) void decode_scores_valu_kernel(const ScoreArgs A) {
  constexpr bool DENSE = MODE == kAllPages, GROUPED = MODE != kPerHead;
  extern __shared__ int pre_lds[];
  __shared__ int wsum[kScoreWaves];
  const T* q = (const T*)A.q;
  const T* k_pool = (const T*)A.k_pool;
  const int P = A.P, Hq = A.Hq, Hkv = A.Hkv;
  const int lane = threadIdx.x & 63, w = uniform(threadIdx.x >> 6);
  const int gp = pmax_pages(P);
  const int r = lane >> 4, c = lane & 15;
  if (!PRE_GLOBAL)
    block_exclusive_prefix<kScoreThreads>(A.U, [&](int u) { return (unit_slots<MODE>(A, u) + gp - 1) / gp; }, pre_lds, wsum);
  const int* pre = PRE_GLOBAL ? A.pre_g : pre_lds;
  const WaveItems wi = wave_item_range(pre, A.U, w);
  int unit = wi.unit;
  for (int it = wi.begin; it < wi.end; ++it) {
    while (it >= uniform(pre[unit + 1])) ++unit;
    const int grp = it - uniform(pre[unit]);
    const int b = GROUPED ? unit / Hkv : unit / Hq;
    const int hkv = GROUPED ? unit % Hkv : (unit % Hq) / (Hq / Hkv);
    const int hq0 = GROUPED ? hkv * G : unit % Hq;          // first (only) query head of this unit
    const int n = A.seq_lens[b];
    const int n_slots = unit_slots<MODE>(A, unit);
    float coef[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) load8<T>(q + ((size_t)b * Hq + hq0 + g) * kD + 8 * c, coef[g]);
    float wmax[G];
#pragma unroll
    for (int g = 0; g < G; ++g) wmax[g] = -INFINITY;
    for (int pg = 0; pg < gp; ++pg) {
      const int slot = grp * gp + pg;
      if (slot >= n_slots) break;
      const int lp = clampi(DENSE ? slot : A.page_idx[(size_t)unit * A.cap + slot], 0, A.Mmax - 1);
      const int phys = clampi(A.block_table[(size_t)b * A.Mmax + lp], 0, A.n_phys - 1);
      const T* kpage = k_pool + ((size_t)phys * A.HkvPool + hkv) * P * kD + 8 * c;
      for (int s0 = 0; s0 < P / 4; s0 += 16) {          // 16 steps (64 tokens) per sweep of the c lanes
        float zkeep[G];
#pragma unroll
        for (int g = 0; g < G; ++g) zkeep[g] = -INFINITY;
        const int s1 = min(P / 4, s0 + 16);
        for (int s = s0; s < s1; ++s) {
          float x[8];
          load8<T>(kpage + (size_t)(4 * s + r) * kD, x);
          const bool valid = lp * P + 4 * s + r < n;
#pragma unroll
          for (int g = 0; g < G; ++g) {
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc = fmaf(coef[g][i], x[i], acc);
            acc = row16_sum(acc);
            const float z = valid ? A.zscale * acc : -INFINITY;
            if (c == s - s0) zkeep[g] = z;
            wmax[g] = fmaxf(wmax[g], z);
          }
        }
        if (c < s1 - s0) {
#pragma unroll
          for (int g = 0; g < G; ++g) {
            const size_t row = GROUPED ? (size_t)b * Hq + hq0 + g : (size_t)unit;
            A.zbuf[row * A.zstride + (size_t)slot * P + 4 * (s0 + c) + r] = zkeep[g];
          }
        }
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float m = wmax[g];                                   // equal over the 16 lanes of a row
      m = fmaxf(m, __shfl_xor(m, 16));
      m = fmaxf(m, __shfl_xor(m, 32));
      const size_t row = GROUPED ? (size_t)b * Hq + hq0 + g : (size_t)unit;
      if (lane == 0) A.pmax[row * A.n_chunks_max + grp] = m;
    }
  }
}

// bf16 pages with P in {16, 32, 64}: matrix-core path.  Many resident wavefronts with little in flight each stream
// better than few with much: the kernel is compiled for eight wavefronts per SIMD and a wavefront holds two chunks
// of 16 tokens at a time (the next chunk is requested before the current one is consumed).  The page-list and block-table entries
// of up to 64 page slots are resolved at once, one slot per lane (two dependent vector loads per batch of 64 / GP
// items instead of two per page), and handed out with v_readlane.
template <int G, int MODE, int PT, bool PRE_GLOBAL>
__global__ __launch_bounds__(kScoreThreads) __attribute__((amdgpu_waves_per_eu(G <= 4 ? 8 : 6)))
void decode_scores_mfma_kernel(const ScoreArgs A) {
  constexpr bool DENSE = MODE == kAllPages, GROUPED = MODE != kPerHead;
  constexpr int NSET = (G + 3) / 4;
  constexpr int KEEP = PT / 16;                   // 16-token chunks per page
  constexpr int GP = 64 / PT;                     // page slots per item
  constexpr int kBatchItems = 64 / GP;
  extern __shared__ int pre_lds[];
  __shared__ int wsum[kScoreWaves];
  const bf16_t* q = (const bf16_t*)A.q;
  const bf16_t* k_pool = (const bf16_t*)A.k_pool;
  const int Hq = A.Hq, Hkv = A.Hkv;
  const int lane = threadIdx.x & 63, w = uniform(threadIdx.x >> 6);
  const int m = lane & 15, j = lane >> 4;          // MFMA row/column index, K group
  const int kq = m & 3, gl = m >> 2;               // channel quarter; as a row: token of the step,
                                                   // as a column: head within the set
  // row (token gl of the step, quarter kq), K group j -> bytes [gl*256 + (kq*4+j)*16, +16) of the step
  const int lane_off = gl * kD + (kq * 4 + j) * 8;
  if (!PRE_GLOBAL)
    block_exclusive_prefix<kScoreThreads>(A.U, [&](int u) { return (unit_slots<MODE>(A, u) + GP - 1) / GP; }, pre_lds, wsum);
  const int* pre = PRE_GLOBAL ? A.pre_g : pre_lds;
  const WaveItems wi = wave_item_range(pre, A.U, w);
  const int last = (DENSE ? A.Mmax : A.cap) - 1;

  for (int it0 = wi.begin; it0 < wi.end; it0 += kBatchItems) {
    // lane l: page slot l % GP of item it0 + l / GP (clamped to the last item): its unit, logical and physical page
    int l_unit, l_lp, l_phys;
    {
      const int my_it = min(it0 + lane / GP, wi.end - 1);
      int lo = 0, hi = A.U;
      while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (pre[mid] <= my_it) lo = mid; else hi = mid; }
      l_unit = lo;
      const int slot = min((my_it - pre[lo]) * GP + lane % GP, last);
      const int b = GROUPED ? lo / Hkv : lo / Hq;
      l_lp = clampi(DENSE ? slot : A.page_idx[(size_t)lo * A.cap + slot], 0, A.Mmax - 1);
      l_phys = clampi(A.block_table[(size_t)b * A.Mmax + l_lp], 0, A.n_phys - 1);
    }
    const int n_ck = (min(it0 + kBatchItems, wi.end) - it0) * 4;       // 16-token chunks of this batch

    // state of the item being consumed (wave-uniform), refreshed at its first chunk
    int n = 0, n_slots = 0, slot0 = 0, grp = 0;
    size_t row0 = 0;
    uint4 bq[NSET];
    float wmax[NSET];
    auto open_item = [&](int pg) {
      const int unit = __builtin_amdgcn_readlane(l_unit, pg);
      const int b = GROUPED ? unit / Hkv : unit / Hq;
      const int hq0 = GROUPED ? (unit % Hkv) * G : unit % Hq;
      grp = it0 + pg / GP - uniform(pre[unit]);
      slot0 = grp * GP;
      row0 = GROUPED ? (size_t)b * Hq + hq0 : (size_t)unit;      // first row of z / pmax written
      n = uniform_load(A.seq_lens + b);
      n_slots = DENSE ? clampi((n + PT - 1) / PT, 0, A.Mmax) : clampi(uniform_load(A.n_sel + unit), 0, A.cap);
#pragma unroll
      for (int s = 0; s < NSET; ++s) {
        const int g = min(4 * s + gl, G - 1);          // columns past the group repeat its last head (not stored)
        bq[s] = *reinterpret_cast<const uint4*>(q + ((size_t)b * Hq + hq0 + g) * kD + kq * 32 + j * 8);
        wmax[s] = -INFINITY;
      }
    };
    // chunk ck of the batch = tokens [16 t, 16 t + 16) of page slot pg = ck / KEEP, t = ck % KEEP
    auto request = [&](int ck, uint4 (&a)[4]) {
      const int pg = ck / KEEP, t = ck % KEEP;
      const int unit = __builtin_amdgcn_readlane(l_unit, pg);
      const int hkv = GROUPED ? unit % Hkv : (unit % Hq) / (Hq / Hkv);
      const int phys = __builtin_amdgcn_readlane(l_phys, pg);
      const bf16_t* kc = k_pool + (((size_t)phys * A.HkvPool + hkv) * PT + 16 * t) * kD + lane_off;
#pragma unroll
      for (int s = 0; s < 4; ++s) a[s] = *reinterpret_cast<const uint4*>(kc + s * 4 * kD);
    };
    auto consume = [&](int ck, const uint4 (&a)[4]) {
      const int pg = ck / KEEP, t = ck % KEEP;
      const int slot = slot0 + pg % GP;
      const bool slot_ok = slot < n_slots;             // wave-uniform
      const int tok0 = __builtin_amdgcn_readlane(l_lp, pg) * PT + 16 * t + j;
      float zkeep[NSET];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        // result rows 4j..4j+3 belong to token j of the step
        const bool valid = slot_ok && tok0 + 4 * s < n;
#pragma unroll
        for (int cs = 0; cs < NSET; ++cs) {
          const f32x4_t zero = {0.f, 0.f, 0.f, 0.f};
          const f32x4_t c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a[s]),
                                                                    __builtin_bit_cast(bf16x8_t, bq[cs]), zero, 0, 0, 0);
          const float v01 = (kq & 1) ? c[1] : c[0], v23 = (kq & 1) ? c[3] : c[2];   // c[kq] in two selects
          float v = (kq & 2) ? v23 : v01;
          v += dpp_move<0xB1>(v);
          v += dpp_move<0x4E>(v);
          const float z = valid ? A.zscale * v : -INFINITY;
          if (s == kq) zkeep[cs] = z;                  // lane (j, head, kq) keeps token 4 kq + j of the chunk
          wmax[cs] = fmaxf(wmax[cs], z);
        }
      }
      if (slot_ok) {
#pragma unroll
        for (int cs = 0; cs < NSET; ++cs) {
          const int g = 4 * cs + gl;
          if (g < G) A.zbuf[(row0 + g) * A.zstride + (size_t)slot * PT + 16 * t + 4 * kq + j] = zkeep[cs];
        }
      }
      if (ck % 4 == 3) {                               // last chunk of the item: its maximum
#pragma unroll
        for (int cs = 0; cs < NSET; ++cs) {
          float mx = wmax[cs];                         // equal over the four kq lanes of a head
          mx = fmaxf(mx, __shfl_xor(mx, 16));
          mx = fmaxf(mx, __shfl_xor(mx, 32));
          const int g = 4 * cs + gl;
          if (j == 0 && kq == 0 && g < G) A.pmax[(row0 + g) * A.n_chunks_max + grp] = mx;
        }
      }
    };

    // two chunks in flight, alternating register sets (n_ck is a multiple of 4).  Loads return in issue order, so the
    // query of a new item (every fourth chunk) is requested BEFORE the next chunk's K loads: waiting for it then
    // leaves those in flight.
    // Every request in the loop is unconditional (a load behind a branch makes the wait at the join drain the queue);
    // the last pair of chunks is taken after the loop.
    uint4 a0[4], a1[4];
    request(0, a0);
    int ck = 0;
    for (; ck + 2 < n_ck; ck += 2) {
      if (ck % 4 == 0) open_item(ck / KEEP);
      __builtin_amdgcn_sched_barrier(0);
      request(ck + 1, a1);
      __builtin_amdgcn_sched_barrier(0);
      consume(ck, a0);
      request(ck + 2, a0);
      __builtin_amdgcn_sched_barrier(0);
      consume(ck + 1, a1);
    }
    if (ck % 4 == 0) open_item(ck / KEEP);
    __builtin_amdgcn_sched_barrier(0);
    request(ck + 1, a1);
    __builtin_amdgcn_sched_barrier(0);
    consume(ck, a0);
    consume(ck + 1, a1);
  }
}

// ------------------------------------------------------------------------------------------
// pass 1b (long rows only): multi-workgroup candidate filter
// ------------------------------------------------------------------------------------------
// One workgroup of the solve cannot stream a row of a million scores, and it does not have to: the
// maxima of the 64-token groups written by pass 1 already bound tau from below.
//   level   (one workgroup per row): row maximum from the group maxima, then a 64-bin count histogram of
//           the group maxima above zmax-1.  Every counted group holds at least one score (its maximum)
//           in that bin, and an entry of bin g lies at least (g-i) bins above grid point i, so the counts
//           give a lower bound of the mass at every grid point; the highest grid point whose bound is >= 1
//           is a certified lower bound of tau.  Reads 4 bytes per 64 tokens.
//   compact (slices of kFilterSliceChunks groups x rows): only groups whose maximum exceeds that bound are
//           read (a few hundred per row); their scores above the bound are written out in order.
// The solve then gathers the survivors of all slices into LDS.

// Counts per bin above a base point give a lower bound of the mass at every grid point i.  Returns the
// highest i in [0, 64) whose bound sum_{g > i} cnt[g] * ((g - i - 0.02) * step)^beta reaches 1 (with a
// margin), or 0.  Called by all 1024 threads of a workgroup: 16 lanes per grid point, a DPP row sum, one
// barrier; `flags` is LDS [64].
template <int NB>
__device__ __forceinline__ int certified_level(const int* cnt, float step, float beta, int ibeta, int* flags) {
  const int i = threadIdx.x >> 4, l = threadIdx.x & 15;
  float lb = 0.f;
#pragma unroll
  for (int g = l; g < NB; g += 16)
    if (g > i) lb += (float)cnt[g] * pow_beta(((float)(g - i) - 0.02f) * step, beta, ibeta);
  lb = row16_sum(lb);
  if (l == 0) flags[i] = lb >= 1.0001f ? 1 : 0;
  __syncthreads();
  const uint64_t okm = __ballot(flags[threadIdx.x & 63] != 0);
  return okm ? 63 - __clzll(okm) : 0;
}

constexpr int kFilterThreads = 1024;
constexpr int kFilterWaves = kFilterThreads / 64;
constexpr int kFilterWaveChunks = kFilterSliceChunks / kFilterWaves;   // groups per wavefront: 32
static_assert(kFilterWaveChunks <= 64, "one ballot covers a wavefront's groups");

struct FilterArgs {
  const int32_t* seq_lens; const int32_t* n_sel; const float* zbuf; const float* pmax;
  int32_t* fcount; float* frow; float* flist_u; int32_t* flist_pos;
  int Hq, Hkv, grouped, P, n_slices_max, max_slots, n_chunks_max;
  size_t zstride;
  float beta; int ibeta;
};

template <bool DENSE>
__device__ __forceinline__ int filter_n_slots(const FilterArgs& A, int row) {
  const int lrow = A.grouped ? (row / A.Hq) * A.Hkv + (row % A.Hq) / (A.Hq / A.Hkv) : row;
  const int slots = DENSE ? (A.seq_lens[row / A.Hq] + A.P - 1) / A.P : A.n_sel[lrow];
  return clampi(slots, 0, A.max_slots);
}

template <bool DENSE>
__global__ __launch_bounds__(kFilterThreads) void filter_level_kernel(const FilterArgs A) {
  __shared__ float red[kFilterWaves];
  __shared__ int hist[64];
  __shared__ int flags[64];
  const int row = blockIdx.x, tid = threadIdx.x;
  const int gp = pmax_pages(A.P);
  const int n_chunks = (filter_n_slots<DENSE>(A, row) + gp - 1) / gp;
  if (n_chunks <= kPreGroups) return;                         // short row: the solve reads its group maxima itself
  const float* pm = A.pmax + (size_t)row * A.n_chunks_max;
  float mx = -INFINITY;
  for (int i0 = 0; i0 < n_chunks; i0 += kFilterThreads * 16) {
    float v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = pm[min(i0 + k * kFilterThreads + tid, n_chunks - 1)];
#pragma unroll
    for (int k = 0; k < 16; ++k) mx = fmaxf(mx, v[k]);        // clamped repeats do not change a maximum
  }
  if (tid < 64) hist[tid] = 0;
  const float zmax = block_max(mx, red);
  if (!(zmax > -INFINITY)) {                                  // empty row, or nothing but masked tokens
    if (tid == 0) { A.frow[2 * row] = -INFINITY; A.frow[2 * row + 1] = 0.f; }
    return;
  }
  const float thr0 = zmax - 1.0f - 4e-6f * fmaxf(1.f, fabsf(zmax));
  const float width = zmax - thr0, step = width * (1.0f / 64.0f), inv_step = 64.0f / width;
  for (int i0 = 0; i0 < n_chunks; i0 += kFilterThreads * 16) {
    float v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = pm[min(i0 + k * kFilterThreads + tid, n_chunks - 1)];
#pragma unroll
    for (int k = 0; k < 16; ++k)
      if (i0 + k * kFilterThreads + tid < n_chunks && v[k] > thr0)
        atomicAdd(&hist[min(63, (int)((v[k] - thr0) * inv_step))], 1);
  }
  __syncthreads();
  int level = certified_level<64>(hist, step, A.beta, A.ibeta, flags);
  float thr = thr0 + (float)level * step;
  // A flat row crowds its group maxima into the last few steps below the maximum, and most groups still pass: the
  // same certificate on a histogram of [bound, maximum] resolves them (twice at most).
  for (int refine = 0; refine < 2; ++refine) {
    int above = 0;
    for (int g = level; g < 64; ++g) above += hist[g];
    if (above <= 1024) break;
    __syncthreads();                                          // every thread has read the counts
    const float w2 = zmax - thr, step2 = w2 * (1.0f / 64.0f), inv_step2 = 64.0f / w2;
    if (tid < 64) hist[tid] = 0;
    __syncthreads();
    for (int i0 = 0; i0 < n_chunks; i0 += kFilterThreads * 16) {
      float v[16];
#pragma unroll
      for (int k = 0; k < 16; ++k) v[k] = pm[min(i0 + k * kFilterThreads + tid, n_chunks - 1)];
#pragma unroll
      for (int k = 0; k < 16; ++k)
        if (i0 + k * kFilterThreads + tid < n_chunks && v[k] > thr)
          atomicAdd(&hist[min(63, (int)((v[k] - thr) * inv_step2))], 1);
    }
    __syncthreads();
    level = certified_level<64>(hist, step2, A.beta, A.ibeta, flags);
    if (level == 0) break;
    thr += (float)level * step2;
  }
  if (tid == 0) { A.frow[2 * row] = zmax; A.frow[2 * row + 1] = thr; }
}

// Scores of up to four groups of a wavefront at once (lane = token of the group), -inf where masked.
__device__ __forceinline__ void filter_group_scores(const float* zr, const int (&chunk)[4], int n_valid, int ct,
                                                    int n_cand, float (&z)[4]) {
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int k = 0; k < 4; ++k) z[k] = zr[min(chunk[min(k, n_valid - 1)] * ct + min(lane, ct - 1), n_cand - 1)];
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (k >= n_valid || lane >= ct || chunk[k] * ct + lane >= n_cand) z[k] = -INFINITY;
}

template <bool DENSE>
__global__ __launch_bounds__(kFilterThreads) void filter_compact_kernel(const FilterArgs A) {
  __shared__ int wtot[kFilterWaves];
  const int row = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t lt = (1ull << lane) - 1ull;
  const int gp = pmax_pages(A.P), ct = gp * A.P;              // tokens per group (<= 64)
  const int n_slots = filter_n_slots<DENSE>(A, row);
  const int n_cand = n_slots * A.P, n_chunks = (n_slots + gp - 1) / gp;
  const int c0 = slice * kFilterSliceChunks;
  if (c0 >= n_chunks || n_chunks <= kPreGroups) return;      // past the row's end, or a short row (see the level pass)
  const float zmax = A.frow[2 * row], thr = A.frow[2 * row + 1];
  const float* zr = A.zbuf + (size_t)row * A.zstride;
  const float* pm = A.pmax + (size_t)row * A.n_chunks_max;
  // groups of this wavefront whose maximum can hold a survivor
  const int cw = c0 + w * kFilterWaveChunks;
  const float pmv = pm[min(cw + min(lane, kFilterWaveChunks - 1), n_chunks - 1)];
  const uint64_t pass = __ballot(lane < kFilterWaveChunks && cw + lane < n_chunks && pmv > thr);
  int c = 0;
  for (uint64_t m = pass; m != 0;) {
    int chunk[4], nv = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (m != 0) { chunk[k] = cw + __builtin_ctzll(m); m &= m - 1; ++nv; } else chunk[k] = cw;
    float z[4];
    filter_group_scores(zr, chunk, nv, ct, n_cand, z);
#pragma unroll
    for (int k = 0; k < 4; ++k) c += __popcll(__ballot(z[k] > thr));
  }
  if (lane == 0) wtot[w] = c;
  __syncthreads();
  int off = 0, tot = 0;
  for (int i = 0; i < kFilterWaves; ++i) { const int ci = wtot[i]; if (i < w) off += ci; tot += ci; }
  if (tid == 0) A.fcount[(size_t)row * A.n_slices_max + slice] = tot;
  if (c == 0) return;
  float* lu = A.flist_u + ((size_t)row * A.n_slices_max + slice) * kFilterSliceCap;
  int32_t* lp = A.flist_pos + ((size_t)row * A.n_slices_max + slice) * kFilterSliceCap;
  for (uint64_t m = pass; m != 0;) {                          // second sweep (from cache): ordered write
    int chunk[4], nv = 0;
#pragma unroll
    for (int k = 0; k < 4; ++k)
      if (m != 0) { chunk[k] = cw + __builtin_ctzll(m); m &= m - 1; ++nv; } else chunk[k] = cw;
    float z[4];
    filter_group_scores(zr, chunk, nv, ct, n_cand, z);
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const bool in = z[k] > thr;
      const uint64_t mk = __ballot(in);
      const int o = off + __popcll(mk & lt);
      if (in && o < kFilterSliceCap) { lu[o] = z[k] - zmax; lp[o] = chunk[k] * ct + lane; }
      off += __popcll(mk);
    }
  }
}

// ------------------------------------------------------------------------------------------
// pass 2: threshold, probabilities, weighted value sum
// ------------------------------------------------------------------------------------------
struct SolveShared {
  float list_u[kListCap];         // z - zmax of the candidates that can be in the support
  int32_t list_pos[kListCap];     // their position in the candidate order
  uint32_t list_row[kListCap];    // their V row: (phys*Hkv + hkv)*P + tok
  float obuf[kSolveWaves][kD];
  float red[2][kSolveWaves][3];
  int wcount[2][kSolveWaves];
  float red1[kSolveWaves];
  int hist[64];                   // candidates per 1/64 slice of [thr, zmax] (threshold tightening)
  int flags[64];
};

// Candidate source: the compacted list (in LDS, or the row's overflow list in the workspace), or the score row itself.
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
  for (int i0 = threadIdx.x; i0 < src.n; i0 += 8 * kSolveThreads) {     // eight loads in flight per thread
    float u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) u[j] = src.get_u(min(i0 + j * kSolveThreads, src.n - 1));
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float x = i0 + j * kSolveThreads < src.n ? u[j] - tau : -1.f;
      if (x > 0.f) { f += pow_beta(x, beta, ibeta); d += pow_beta_m1(x, beta, ibeta); ++c; }
    }
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

// Root of sum (u - tau)_+^beta = 1 for u <= 0 with max u = 0: tau in [lo_init, 0), where lo_init >= -1
// is any point with mass >= 1.
// Safeguarded iteration inside a bracket [lo,hi], F(lo) >= 1 > F(hi).  From a left point the step is
// the exact root for the current support when beta is 1 or 2 (closed forms), Newton otherwise; from a
// right point a Newton step (F is convex, so it lands left of the root).  For beta in {1,2} the root is
// accepted as exact once a closed-form step leaves the support count unchanged.
// `eval(tau, F, D, cnt)` evaluates the mass, its negated derivative and the support count at tau.
// `seed`: where to take the first evaluation if it lies inside the bracket (NaN: none); `evals` counts
// the evaluations.
template <typename Eval>
__device__ __forceinline__ float solve_tau_core(Eval&& eval, float lo_init, float seed, int ibeta, int& supp,
                                                int& evals) {
  float lo = lo_init, hi = 0.f;
  float tau = (seed > lo && seed < hi) ? seed : lo;
  int pending_cnt = -1;
  int cnt = 0;
  bool reeval = false;
  evals = 0;
  for (int it = 0; it < 64; ++it) {
    float F, D;
    eval(tau, F, D, cnt);
    ++evals;
    if (pending_cnt >= 0 && cnt == pending_cnt) break;       // exact step kept the support: done
    if (fabsf(F - 1.0f) <= 4e-7f) break;                     // float32 resolution of F: tau is the root
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
    if (next == tau) break;                                  // no representable progress
    if (!(next > lo && next < hi)) { next = 0.5f * (lo + hi); pending_cnt = -1; }
    if (hi - lo <= 1.2e-7f || (pending_cnt < 0 && fabsf(next - tau) <= 6e-8f)) { tau = next; reeval = true; break; }
    tau = next;
  }
  if (reeval) {                                              // tau moved after the last evaluation
    float F, D;
    eval(tau, F, D, cnt);
    ++evals;
  }
  supp = cnt;
  return tau;
}

// The whole workgroup iterates (one barrier per evaluation).
template <typename Src>
__device__ __forceinline__ float solve_tau(const Src& src, float lo_init, float seed, float beta, int ibeta,
                                           SolveShared& sh, int& supp, int& evals) {
  int parity = 0;
  return solve_tau_core([&](float tau, float& F, float& D, int& cnt) {
    eval_mass(src, tau, beta, ibeta, sh, parity, F, D, cnt);
    parity ^= 1;
  }, lo_init, seed, ibeta, supp, evals);
}

// Short candidate lists (at most kWaveList entries, the usual case once the certified bound has been
// applied): one wavefront holds them in registers and iterates without any barrier; the result is handed
// to the other wavefronts through LDS.  Called by the whole workgroup.
constexpr int kWaveList = 256;
// entries of one wavefront in registers (u[k] of lane l is list entry l + 64 k, -inf past the end)
__device__ __forceinline__ float solve_tau_regs(const float (&u)[kWaveList / 64], float lo_init, float seed, float beta,
                                                int ibeta, int& supp, int& evals) {
  return solve_tau_core([&](float t, float& F, float& D, int& cnt) {
    float f = 0.f, d = 0.f; int c = 0;
#pragma unroll
    for (int k = 0; k < kWaveList / 64; ++k) {
      const float x = u[k] - t;
      if (x > 0.f) { f += pow_beta(x, beta, ibeta); d += pow_beta_m1(x, beta, ibeta); ++c; }
    }
    F = wave_sum(f); D = beta * wave_sum(d); cnt = wave_sum_i(c);
  }, lo_init, seed, ibeta, supp, evals);
}
__device__ __forceinline__ float solve_tau_wave(const float* list_u, int n, float lo_init, float seed, float beta,
                                                int ibeta, SolveShared& sh, int& supp, int& evals) {
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    float u[kWaveList / 64];
#pragma unroll
    for (int k = 0; k < kWaveList / 64; ++k) u[k] = lane + 64 * k < n ? list_u[lane + 64 * k] : -INFINITY;
    int sp = 0, ev = 0;
    const float tau = solve_tau_regs(u, lo_init, seed, beta, ibeta, sp, ev);
    if (lane == 0) { sh.red1[0] = tau; sh.wcount[0][0] = sp; sh.wcount[0][1] = ev; }
  }
  __syncthreads();
  supp = sh.wcount[0][0];
  evals = sh.wcount[0][1];
  return sh.red1[0];
}

struct SolveArgs {
  const void* v_pool;
  const int32_t* block_table; const int32_t* seq_lens; const int32_t* page_idx; const int32_t* n_sel;
  const float* zbuf; const float* pmax;
  float* out; float* tau_out; int32_t* supp_out;
  ekv_decode_extras ex;
  int Hq, Hkv, P, Mmax, cap, n_chunks_max, n_phys;
  size_t zstride;
  float a, beta; int ibeta;
  // results of the filter passes (null for short rows)
  const int32_t* fcount; const float* frow; const float* flist_u; const int32_t* flist_pos; int n_slices_max;
  int grouped;
  int HkvPool;
  // per-row overflow list in the workspace for candidate lists beyond the LDS list (null / 0 when rows cannot have one)
  float* spill_u; int32_t* spill_pos; int spill_cap;
};

// V row index (phys*Hkv + hkv)*P + tok of candidate position `pos`.
template <bool DENSE>
__device__ __forceinline__ uint32_t v_row_of(const SolveArgs& A, int b, int bh, int hkv, int pos) {
  const int slot = pos / A.P, tok = pos - slot * A.P;
  const int lp = DENSE ? slot : clampi(A.page_idx[(size_t)bh * A.cap + slot], 0, A.Mmax - 1);
  const int phys = clampi(A.block_table[(size_t)b * A.Mmax + lp], 0, A.n_phys - 1);
  return (uint32_t)((phys * A.HkvPool + hkv) * A.P + tok);
}
template <bool DENSE>
__device__ __forceinline__ int token_of(const SolveArgs& A, int bh, int pos) {
  const int slot = pos / A.P, tok = pos - slot * A.P;
  const int lp = DENSE ? slot : A.page_idx[(size_t)bh * A.cap + slot];
  return lp * A.P + tok;
}

// Final reduction of the per-lane partial outputs (acc[8] = channels 8c..8c+7 of a row slot).
__device__ __forceinline__ void reduce_output(float (&acc)[8], SolveShared& sh, float* __restrict__ out) {
  const int tid = threadIdx.x, c = tid & 15, w = tid >> 6;
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
    out[tid] = s;
  }
}

// Weighted sum of the V rows of the `tot` support entries in LDS (weight list_u[e], row list_row[e]): 64 row
// slots x 16 lanes, eight independent 16-byte loads in flight per lane (clamped entries carry weight 0).  A row
// slot adds its entries in ascending order.
template <typename T>
__device__ __forceinline__ void gather_support(const T* __restrict__ v_pool, const SolveShared& sh, int tot, float (&acc)[8]) {
  const int rs = threadIdx.x >> 4, c = threadIdx.x & 15;
  constexpr int kSlots = kSolveThreads / 16;
  for (int e0 = 0; e0 < tot; e0 += 8 * kSlots) {
    Raw8<T> vr[8]; float pw[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int e = e0 + kSlots * j + rs;
      const int ec = min(e, tot - 1);
      pw[j] = e < tot ? sh.list_u[ec] : 0.f;
      load_raw8(v_pool + (size_t)sh.list_row[ec] * kD + 8 * c, vr[j]);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float vv[8];
      widen8(vr[j], vv);
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] = fmaf(pw[j], vv[i], acc[i]);
    }
  }
}

template <typename T, bool DENSE>
__global__ __launch_bounds__(kSolveThreads) void decode_solve_kernel(const SolveArgs A) {
  __shared__ SolveShared sh;
  const int Hq = A.Hq, Hkv = A.Hkv, P = A.P;
  const int bh = blockIdx.x, b = bh / Hq, hq = bh % Hq, hkv = hq / (Hq / Hkv);
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t lt = (1ull << lane) - 1ull;
  const T* v_pool = (const T*)A.v_pool;
  const int n = A.seq_lens[b];
  const int lrow = A.grouped ? b * Hkv + hkv : bh;          // row of the page list this head reads
  const int n_slots = clampi(DENSE ? (n + P - 1) / P : A.n_sel[lrow], 0, DENSE ? A.Mmax : A.cap);
  const int n_cand = n_slots * P;
  const int n_chunks = (n_slots + pmax_pages(P) - 1) / pmax_pages(P);
  const int chunk_tokens = pmax_pages(P) * P;
  const float* zr = A.zbuf + (size_t)bh * A.zstride;
  const float* pm = A.pmax + (size_t)bh * A.n_chunks_max;
  const float beta = A.beta; const int ibeta = A.ibeta;
  float* out = A.out + (size_t)bh * kD;

  // warm start (optional): requested with the first loads, used once zmax is known
  const float seed_z = A.ex.tau_seed != nullptr ? A.ex.tau_seed[bh] : NAN;
  float zmax, thr_f = 0.f;
  // Rows of at most kPreGroups groups: thread t holds the maxima of the gpt consecutive groups gpt*t .. gpt*t+gpt-1
  // (gpt = 1 up to 1024 groups)
  float mypm[kPreR];
#pragma unroll
  for (int k = 0; k < kPreR; ++k) mypm[k] = -INFINITY;
  const bool pre = n_chunks <= kPreGroups;
  const int gpt = (n_chunks + kSolveThreads - 1) / kSolveThreads;
  // The filter passes are launched when the list CAPACITY allows longer rows than that; whether this row took them
  // is decided here, from its actual length (they leave shorter rows alone).
  const bool filt = A.fcount != nullptr && !pre;
  if (filt) {
    zmax = n_cand > 0 ? A.frow[2 * bh] : -INFINITY;
    thr_f = n_cand > 0 ? A.frow[2 * bh + 1] : 0.f;
  } else if (pre) {
    float mx = -INFINITY;
#pragma unroll
    for (int k = 0; k < kPreR; ++k) {
      const int g = gpt * tid + k;
      if (k < gpt && g < n_chunks) { mypm[k] = pm[g]; mx = fmaxf(mx, mypm[k]); }
    }
    zmax = block_max(mx, sh.red1);
  } else {
    float mx = -INFINITY;
    for (int i = tid; i < n_chunks; i += kSolveThreads) mx = fmaxf(mx, pm[i]);
    zmax = block_max(mx, sh.red1);
  }
  if (!(zmax > -INFINITY)) {                // no valid candidate at all
    if (tid < kD) out[tid] = 0.f;
    if (tid == 0) {
      A.tau_out[bh] = INFINITY; A.supp_out[bh] = 0;
      if (A.ex.solve_evals != nullptr) A.ex.solve_evals[bh] = 0;
      if (A.ex.tau_ref != nullptr && A.ex.kept_mass_ref != nullptr) A.ex.kept_mass_ref[bh] = 0.f;
      if (A.ex.tau_ref != nullptr && A.ex.kept_supp_ref != nullptr) A.ex.kept_supp_ref[bh] = 0;
      if (DENSE && A.ex.lse != nullptr) A.ex.lse[bh] = -INFINITY;
    }
    return;
  }
  // Only z > zmax - 1 can be in the support.  That set is compacted IN ORDER into LDS in rounds of
  // kRoundTokens candidates: wavefront w of a round owns 64*kRoundLoads consecutive positions, so
  // (round, w, load, lane) order is candidate order.  A 64-position load whose chunk maximum is <= thr is
  // not issued.  The same pass histograms the candidates over 64 slices of [thr, zmax]; counts alone give
  // a lower bound of the mass at every slice boundary (an entry of slice j lies at least j-i slices above
  // boundary i), hence a tighter valid threshold: it becomes the starting point of the solve, and, if the
  // candidates did not fit in LDS, the threshold of one more compaction pass.
  float thr = filt ? thr_f : zmax - 1.0f - 4e-6f * fmaxf(1.f, fabsf(zmax));
  // Short rows: the group maxima (held by the threads) give a first certified bound of tau -- every group
  // counted in a bin holds at least its maximum there -- and only the groups whose maximum exceeds it are
  // read at all: their scores are fetched through an ordered list of group numbers, so that a row of any
  // length up to kPreGroups groups normally takes one round of loads.
  if (pre) {
    const float step = (zmax - thr) * (1.0f / 64.0f), inv_step = 64.0f / (zmax - thr);
    if (tid < 64) sh.hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPreR; ++k)
      if (k < gpt && mypm[k] > thr) atomicAdd(&sh.hist[min(63, (int)((mypm[k] - thr) * inv_step))], 1);
    __syncthreads();
    thr += (float)certified_level<64>(sh.hist, step, beta, ibeta, sh.flags) * step;
    if (A.ex.tau_seed != nullptr) {
      // A seed above that bound becomes the candidate threshold if the group maxima alone already put a
      // mass of 1 above it (then the full mass there is >= 1, i.e. the seed is a lower bound of tau).
      const bool try_seed = seed_z > thr && seed_z < zmax;            // false for NaN
      float f = 0.f;
#pragma unroll
      for (int k = 0; k < kPreR; ++k)
        if (try_seed && mypm[k] > seed_z) f += pow_beta(mypm[k] - seed_z, beta, ibeta);
      f = block_sum(f, sh.red1);
      if (try_seed && f >= 1.0001f) thr = seed_z;
    }
  }
  const float seed_u = seed_z - zmax;
  int evals = 0;
  float lo_u = thr - zmax;
  // chunk skipping pays only when there is a lot to skip (dense rows); short candidate lists are read whole,
  // which saves the dependent load of the chunk maxima in every round
  const bool can_skip = (chunk_tokens & 63) == 0 && n_cand > 4 * kRoundTokens;
  int n_list = 0, parity = 0;
  bool in_lds = true;
  bool in_spill = false;          // the candidate list outgrew LDS and lives in this row's overflow list
  bool prefilled = false;
  float* const su = A.spill_u != nullptr ? A.spill_u + (size_t)bh * A.spill_cap : nullptr;
  int32_t* const sp = A.spill_pos != nullptr ? A.spill_pos + (size_t)bh * A.spill_cap : nullptr;
  if (filt) {
    // survivors of the filter passes: gather the per-slice lists, in slice order, if they fit
    const int n_slices = (n_chunks + kFilterSliceChunks - 1) / kFilterSliceChunks;
    const int cs = tid < n_slices ? A.fcount[(size_t)bh * A.n_slices_max + tid] : 0;
    int inc = cs;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) { const int t = __shfl_up(inc, d); if (lane >= d) inc += t; }
    if (lane == 63) sh.wcount[0][w] = inc;
    const int bad = __syncthreads_or(cs > kFilterSliceCap);
    int base = 0, tot = 0;
    for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[0][i]; if (i < w) base += ci; tot += ci; }
    if (!bad && tot <= kListCap) {
      int* start = reinterpret_cast<int*>(sh.list_row);      // free until the solve is done
      if (tid < n_slices) { start[2 * tid] = base + inc - cs; start[2 * tid + 1] = cs; }
      __syncthreads();
      for (int sl = w; sl < n_slices; sl += kSolveWaves) {
        const int o0 = start[2 * sl], cnt = start[2 * sl + 1];
        const float* lu = A.flist_u + ((size_t)bh * A.n_slices_max + sl) * kFilterSliceCap;
        const int32_t* lp = A.flist_pos + ((size_t)bh * A.n_slices_max + sl) * kFilterSliceCap;
        for (int e = lane; e < cnt; e += 64) { sh.list_u[o0 + e] = lu[e]; sh.list_pos[o0 + e] = lp[e]; }
      }
      n_list = tot;
      prefilled = true;
      lo_u = fminf(thr - zmax, -1e-7f);
    } else if (!bad && su != nullptr && tot <= A.spill_cap) {
      // too many survivors for LDS: concatenate the per-slice lists, in slice order, into the row's overflow list
      int* start = reinterpret_cast<int*>(sh.list_row);
      if (tid < n_slices) { start[2 * tid] = base + inc - cs; start[2 * tid + 1] = cs; }
      __syncthreads();
      for (int sl = w; sl < n_slices; sl += kSolveWaves) {
        const int o0 = start[2 * sl], cnt = start[2 * sl + 1];
        const float* lu = A.flist_u + ((size_t)bh * A.n_slices_max + sl) * kFilterSliceCap;
        const int32_t* lp = A.flist_pos + ((size_t)bh * A.n_slices_max + sl) * kFilterSliceCap;
        for (int e = lane; e < cnt; e += 64) { su[o0 + e] = lu[e]; sp[o0 + e] = lp[e]; }
      }
      n_list = tot;
      prefilled = true;
      in_lds = false; in_spill = true;
      lo_u = fminf(thr - zmax, -1e-7f);
    }
    __syncthreads();
  }
  if (pre) {
    // ordered list of the groups above the bound: thread t owns consecutive groups, so (thread, k) order is group order
    int* glist = reinterpret_cast<int*>(sh.list_row);        // free until the solve is done
    int n_pass = 0;
    for (int refine = 0;; ++refine) {
    int goff;
    n_pass = 0;
    if (gpt == 1) {                                          // one group per thread (rows up to 65 536 tokens): a ballot
      const bool gp = mypm[0] > thr;
      const uint64_t gmk = __ballot(gp);
      if (lane == 0) sh.wcount[parity][w] = __popcll(gmk);
      __syncthreads();
      goff = 0;
      for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) goff += ci; n_pass += ci; }
      if (gp) glist[goff + __popcll(gmk & lt)] = tid;
    } else {
      int mine = 0;
#pragma unroll
      for (int k = 0; k < kPreR; ++k) mine += mypm[k] > thr ? 1 : 0;
      int inc = mine;
#pragma unroll
      for (int dlt = 1; dlt < 64; dlt <<= 1) { const int t = __shfl_up(inc, dlt); if (lane >= dlt) inc += t; }
      if (lane == 63) sh.wcount[parity][w] = inc;
      __syncthreads();
      goff = inc - mine;
      for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) goff += ci; n_pass += ci; }
#pragma unroll
      for (int k = 0; k < kPreR; ++k)
        if (mypm[k] > thr) glist[goff++] = gpt * tid + k;
    }
    parity ^= 1;
    n_pass = __builtin_amdgcn_readfirstlane(n_pass);
    __syncthreads();
    // The usual row is done here: a few dozen groups pass.  A flat row, where most groups still pass, has its group
    // maxima crowded into the last few of the 64 steps below the maximum; the same certificate on a histogram of
    // [bound, maximum] resolves them (twice at most: 1/64^3 of the first width), and the list is rebuilt.
    if (__builtin_expect(n_pass <= kSolveWaves * kRoundLoads || refine == 2, 1)) break;
    const float step2 = (zmax - thr) * (1.0f / 64.0f), inv_step2 = 64.0f / (zmax - thr);
    if (tid < 64) sh.hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kPreR; ++k)
      if (k < gpt && mypm[k] > thr) atomicAdd(&sh.hist[min(63, (int)((mypm[k] - thr) * inv_step2))], 1);
    __syncthreads();
    const int level2 = certified_level<64>(sh.hist, step2, beta, ibeta, sh.flags);
    if (level2 == 0) break;
    thr += (float)level2 * step2;
    }
    // wavefront w of a round owns `per` consecutive list entries: (round, w, load, lane) is candidate order
    constexpr int kRoundGroups = kSolveWaves * kRoundLoads;
    // second half of a round: mask, count, exchange the counts (one barrier), ordered compaction into the list
    auto compact_round = [&](int j0, float (&v)[kRoundLoads], const int (&vpos)[kRoundLoads]) {
      const int rem = min(n_pass - j0, kRoundGroups);
      const int per = (rem + kSolveWaves - 1) / kSolveWaves;
      const int jw = j0 + w * per, jend = j0 + rem;
      int c = 0;
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) {
        const bool ok = i < per && jw + i < jend && lane < chunk_tokens && vpos[i] < n_cand;
        v[i] = ok ? v[i] : -INFINITY;
        c += __popcll(__ballot(v[i] > thr));
      }
      if (lane == 0) sh.wcount[parity][w] = c;
      __syncthreads();
      int off = n_list, tot = 0;
      for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) off += ci; tot += ci; }
      n_list += tot;
      parity ^= 1;
      if (__builtin_expect(in_lds && n_list > kListCap, 0)) {
        // The list outgrows LDS: it continues in the row's overflow list, to which the entries of the earlier rounds
        // move first (the barrier above ordered their LDS writes).
        in_lds = false;
        if (su != nullptr) {
          in_spill = true;
          for (int e = tid; e < n_list - tot; e += kSolveThreads) { su[e] = sh.list_u[e]; sp[e] = sh.list_pos[e]; }
        }
      }
      if (in_spill && n_list > A.spill_cap) in_spill = false;
      auto emit = [&](auto* du, auto* dp) {
#pragma unroll
        for (int i = 0; i < kRoundLoads; ++i) {
          const bool in = v[i] > thr;
          const uint64_t mk = __ballot(in);
          if (in) {
            const int o = off + __popcll(mk & lt);
            du[o] = v[i] - zmax;
            dp[o] = vpos[i];
          }
          off += __popcll(mk);
        }
      };
      if (__builtin_expect(in_lds, 1)) emit(sh.list_u, sh.list_pos);
      else if (in_spill) emit(su, sp);
    };
    for (int j0 = 0; j0 < n_pass; j0 += kRoundGroups) {     // one round in the usual case
      const int rem = min(n_pass - j0, kRoundGroups);
      const int per = (rem + kSolveWaves - 1) / kSolveWaves;
      const int jw = j0 + w * per;
      float v[kRoundLoads]; int vpos[kRoundLoads];
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) {
        v[i] = -INFINITY; vpos[i] = 0;
        if (i < per) {                                   // wave-uniform
          const int g = glist[min(jw + i, n_pass - 1)];
          vpos[i] = g * chunk_tokens + lane;
          v[i] = zr[min(vpos[i], n_cand - 1)];
        }
      }
      compact_round(j0, v, vpos);
    }
    if (in_lds || in_spill) lo_u = fminf(thr - zmax, -1e-7f);
  }
  for (int pass = 0; pass < 3 && !prefilled && !pre; ++pass) {
    const float width = zmax - thr, slice = width * (1.0f / 64.0f), inv_slice = 64.0f / width;
    if (tid < 64) sh.hist[tid] = 0;
    n_list = 0; in_lds = true;
    __syncthreads();
    for (int round0 = 0; round0 < n_cand; round0 += kRoundTokens) {
      const int seg = round0 + w * 64 * kRoundLoads;
      // The chunk maxima of the round are fetched first as one batch (clamped, unconditional), then the
      // score loads of the chunks that can hold a candidate are issued back to back; nothing is consumed
      // before all of them are in flight.
      float pmv[kRoundLoads];
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) pmv[i] = can_skip ? pm[min(seg + i * 64, n_cand - 1) / chunk_tokens] : INFINITY;
      float v[kRoundLoads];
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) {
        const int pos0 = seg + i * 64;
        const float pmu = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(pmv[i])));
        v[i] = -INFINITY;
        if (pos0 < n_cand && (!can_skip || pmu > thr)) v[i] = zr[min(pos0 + lane, n_cand - 1)];
      }
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) v[i] = seg + i * 64 + lane < n_cand ? v[i] : -INFINITY;
      int c = 0;
#pragma unroll
      for (int i = 0; i < kRoundLoads; ++i) {
        const bool in = v[i] > thr;
        c += __popcll(__ballot(in));
        if (in) atomicAdd(&sh.hist[min(63, (int)((v[i] - thr) * inv_slice))], 1);
      }
      if (lane == 0) sh.wcount[parity][w] = c;
      __syncthreads();
      int off = n_list, tot = 0;
      for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) off += ci; tot += ci; }
      n_list += tot;
      parity ^= 1;
      if (n_list > kListCap) in_lds = false;
      if (in_lds) {
#pragma unroll
        for (int i = 0; i < kRoundLoads; ++i) {
          const bool in = v[i] > thr;
          const uint64_t mk = __ballot(in);
          if (in) {
            const int o = off + __popcll(mk & lt);
            sh.list_u[o] = v[i] - zmax;
            sh.list_pos[o] = seg + i * 64 + lane;
          }
          off += __popcll(mk);
        }
      }
    }
    __syncthreads();
    // highest slice boundary whose counted lower bound of the mass is still >= 1
    const int level = certified_level<64>(sh.hist, slice, beta, ibeta, sh.flags);
    const float thr2 = thr + (float)level * slice;
    if (in_lds) { lo_u = fminf(thr2 - zmax, -1e-7f); break; }
    if (level == 0) break;                       // no tighter threshold from counts: stream the row
    thr = thr2;
    lo_u = thr - zmax;
  }
  __syncthreads();

  // Short lists and no side output over all candidates (the usual call): ONE wavefront finishes the row --
  // V rows resolved while it solves in registers, support compacted with ballots, values gathered by its four
  // 16-lane rows -- and the other fifteen leave; nothing below this point needs a barrier then.
  const bool block_extras = (A.ex.tau_ref != nullptr && (A.ex.kept_mass_ref != nullptr || A.ex.kept_supp_ref != nullptr)) ||
                            (DENSE && A.ex.lse != nullptr);
  if (__builtin_expect(in_lds && n_list <= kWaveList && !block_extras, 1)) {
    if (w != 0) return;
    constexpr int KW = kWaveList / 64;
    float u[KW]; int pos[KW]; uint32_t row[KW];
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const int e = lane + 64 * k;
      u[k] = e < n_list ? sh.list_u[e] : -INFINITY;
      pos[k] = e < n_list ? sh.list_pos[e] : 0;
    }
#pragma unroll
    for (int k = 0; k < KW; ++k) row[k] = v_row_of<DENSE>(A, b, lrow, hkv, pos[k]);     // clamped, unconditional
    int supp_w = 0;
    const float tau_w = solve_tau_regs(u, lo_u, seed_u, beta, ibeta, supp_w, evals);
    // ordered compaction of the support: (p, row, position) of entry e = lane + 64 k, k-major = candidate order
    int n_sup = 0;
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < KW; ++k) {
      const float x = u[k] - tau_w;
      const bool in = x > 0.f;
      const uint64_t mk = __ballot(in);
      if (in) {
        const int o = n_sup + __popcll(mk & lt);
        sh.list_u[o] = pow_beta(x, beta, ibeta);
        sh.list_row[o] = row[k];
        sh.list_pos[o] = pos[k];
      }
      n_sup += __popcll(mk);
    }
    __builtin_amdgcn_wave_barrier();
    // weighted value sum: 4 row slots x 16 lanes, batches of 8 independent 16-byte loads per lane
    const int rs = lane >> 4, c = lane & 15;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int e0 = 0; e0 < n_sup; e0 += 32) {
      Raw8<T> vr[8]; float pw[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + 4 * j + rs;
        const int ec = min(e, n_sup - 1);                              // clamped: loads stay unconditional
        pw[j] = e < n_sup ? sh.list_u[ec] : 0.f;
        load_raw8(v_pool + (size_t)sh.list_row[ec] * kD + 8 * c, vr[j]);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float vv[8];
        widen8(vr[j], vv);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = fmaf(pw[j], vv[i], acc[i]);
      }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      acc[i] += __shfl_xor(acc[i], 16);
      acc[i] += __shfl_xor(acc[i], 32);
    }
    if (lane < 16) {
      *reinterpret_cast<float4*>(out + 8 * c) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      *reinterpret_cast<float4*>(out + 8 * c + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
    if (A.ex.support_tokens != nullptr) {
      int32_t* dst = A.ex.support_tokens + (size_t)bh * A.ex.support_cap;
      for (int e = lane; e < n_sup && e < A.ex.support_cap; e += 64) dst[e] = token_of<DENSE>(A, lrow, sh.list_pos[e]);
    }
    if (lane == 0) {
      A.tau_out[bh] = tau_w + zmax; A.supp_out[bh] = supp_w;
      if (A.ex.solve_evals != nullptr) A.ex.solve_evals[bh] = evals;
    }
    return;
  }

  float tau_u; int supp;
  if (in_lds) {
    // V row of every candidate, fetched now (two dependent loads) and consumed after the solve
    uint32_t rowreg[kListCap / kSolveThreads];
#pragma unroll
    for (int k = 0; k < kListCap / kSolveThreads; ++k) {
      const int e = min(tid + k * kSolveThreads, n_list - 1);      // clamped: loads stay unconditional
      rowreg[k] = v_row_of<DENSE>(A, b, lrow, hkv, sh.list_pos[e]);
    }
    const ListSrc ls{sh.list_u, sh.list_pos, n_list};
    if (n_list <= kWaveList) tau_u = solve_tau_wave(sh.list_u, n_list, lo_u, seed_u, beta, ibeta, sh, supp, evals);
    else tau_u = solve_tau(ls, lo_u, seed_u, beta, ibeta, sh, supp, evals);
#pragma unroll
    for (int k = 0; k < kListCap / kSolveThreads; ++k) {
      const int e = tid + k * kSolveThreads;
      if (e < n_list) sh.list_row[e] = rowreg[k];
    }
    __syncthreads();
    // in-place ordered compaction of the support: entry e keeps (p_e, pos_e, row_e)
    int n_sup = 0;
    for (int e0 = 0; e0 < n_list; e0 += kSolveThreads) {
      const int e = e0 + tid;
      const float x = e < n_list ? sh.list_u[e] - tau_u : -1.f;
      const int pe = e < n_list ? sh.list_pos[e] : 0;
      const uint32_t re = e < n_list ? sh.list_row[e] : 0u;
      const bool in = x > 0.f;
      const uint64_t mk = __ballot(in);
      if (lane == 0) sh.wcount[parity][w] = __popcll(mk);
      __syncthreads();                                     // all reads of this block are done
      int off = n_sup, tot = 0;
      for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) off += ci; tot += ci; }
      parity ^= 1;
      if (in) {
        const int o = off + __popcll(mk & lt);
        sh.list_u[o] = pow_beta(x, beta, ibeta);
        sh.list_pos[o] = pe;
        sh.list_row[o] = re;
      }
      n_sup += tot;
    }
    __syncthreads();
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    gather_support<T>(v_pool, sh, n_sup, acc);
    reduce_output(acc, sh, out);
    if (A.ex.support_tokens != nullptr) {
      int32_t* dst = A.ex.support_tokens + (size_t)bh * A.ex.support_cap;
      for (int e = tid; e < n_sup && e < A.ex.support_cap; e += kSolveThreads)
        dst[e] = token_of<DENSE>(A, lrow, sh.list_pos[e]);
    }
  } else {
    // The candidates do not fit in LDS.  They are iterated where they are: in the row's overflow list (every
    // evaluation of the mass reads that list), or -- a row so flat that even that list is too small -- in the score
    // row itself.  The support is then gathered in rounds of 4096 candidates (wavefront w owns 256 consecutive ones):
    // the support tokens of a round are compacted into LDS (weight, V row, position) -- at most 4096, so they always
    // fit -- and their V rows summed by the 64 row slots with batched independent loads.
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    int n_out = 0;
    auto finish = [&](const auto& src) {
      tau_u = solve_tau(src, lo_u, seed_u, beta, ibeta, sh, supp, evals);
      for (int base = 0; base < src.n; base += 4 * kSolveThreads) {
        float xs[4]; int ps[4]; uint32_t rw[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int idx = min(base + w * 256 + i * 64 + lane, src.n - 1);
          xs[i] = src.get_u(idx); ps[i] = src.get_pos(idx);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) rw[i] = v_row_of<DENSE>(A, b, lrow, hkv, min(ps[i], n_cand - 1));   // unconditional
        int cw = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          xs[i] = base + w * 256 + i * 64 + lane < src.n ? xs[i] - tau_u : -1.f;
          cw += __popcll(__ballot(xs[i] > 0.f));
        }
        if (lane == 0) sh.wcount[parity][w] = cw;
        __syncthreads();                                   // also: the previous round's gather is done
        int off = 0, tot = 0;
        for (int i = 0; i < kSolveWaves; ++i) { const int ci = sh.wcount[parity][i]; if (i < w) off += ci; tot += ci; }
        parity ^= 1;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool in = xs[i] > 0.f;
          const uint64_t mk = __ballot(in);
          if (in) {
            const int o = off + __popcll(mk & lt);
            sh.list_u[o] = pow_beta(xs[i], beta, ibeta);
            sh.list_row[o] = rw[i];
            sh.list_pos[o] = ps[i];
          }
          off += __popcll(mk);
        }
        __syncthreads();
        gather_support<T>(v_pool, sh, tot, acc);
        if (A.ex.support_tokens != nullptr) {
          int32_t* dst = A.ex.support_tokens + (size_t)bh * A.ex.support_cap;
          for (int e = tid; e < tot && n_out + e < A.ex.support_cap; e += kSolveThreads)
            dst[n_out + e] = token_of<DENSE>(A, lrow, sh.list_pos[e]);
        }
        n_out += tot;
      }
    };
    if (in_spill) {
      __syncthreads();                                     // the overflow list is complete and visible to the workgroup
      finish(ListSrc{su, sp, n_list});
    } else {
      finish(RowSrc{zr, n_cand, zmax});
    }
    reduce_output(acc, sh, out);
  }
  const float tau = tau_u + zmax;
  if (tid == 0) {
    A.tau_out[bh] = tau; A.supp_out[bh] = supp;
    if (A.ex.solve_evals != nullptr) A.ex.solve_evals[bh] = evals;
  }

  // ---- optional side outputs over ALL candidates ----------------------------------------
  if (A.ex.tau_ref != nullptr && (A.ex.kept_mass_ref != nullptr || A.ex.kept_supp_ref != nullptr)) {
    const float tr = A.ex.tau_ref[bh];
    float f = 0.f; int c = 0;
    for (int i = tid; i < n_cand; i += kSolveThreads) {
      const float x = zr[i] - tr;
      if (x > 0.f) { f += pow_beta(x, beta, ibeta); ++c; }
    }
    f = block_sum(f, sh.red1);
    c = block_sum_i(c, sh.wcount[0]);
    if (tid == 0) {
      if (A.ex.kept_mass_ref != nullptr) A.ex.kept_mass_ref[bh] = f;
      if (A.ex.kept_supp_ref != nullptr) A.ex.kept_supp_ref[bh] = c;
    }
  }
  if (DENSE && A.ex.lse != nullptr) {
    // log sum_j exp(s_j) with s_j = z_j / a, shifted by the maximum
    const float inv_a = 1.0f / A.a;
    float f = 0.f;
    for (int i = tid; i < n_cand; i += kSolveThreads) f += __expf((zr[i] - zmax) * inv_a);
    f = block_sum(f, sh.red1);
    if (tid == 0) A.ex.lse[bh] = zmax * inv_a + __logf(f);
  }
}

// ------------------------------------------------------------------------------------------
// pass 2 for short candidate rows: one wavefront per (b, h)
// ------------------------------------------------------------------------------------------
// Rows of at most 64*KZ candidate tokens (page lists of a few dozen pages): all scores of a row sit in the
// registers of ONE wavefront (lane l holds candidates i*64 + l), the threshold is solved there, and the support
// is gathered through a small LDS list in candidate order, flushed whenever it could overflow -- any support
// size, no barrier.  Four rows per 256-thread workgroup: with hundreds or thousands of rows (many sequences
// of a few thousand tokens) the 1024-thread workgroup per row of the kernel above fills the GPU several times
// over.  Sparse and group-shared lists only.
constexpr int kWaveRowList = 256;        // LDS list entries per wavefront
constexpr int kWaveRowsMin = 512;        // up to 512 rows the workgroup kernel takes one round and is as fast

template <typename T, int KZ>
__global__ __launch_bounds__(256) void decode_solve_wave_kernel(const SolveArgs A, int BH) {
  __shared__ float l_p[4][kWaveRowList];
  __shared__ uint32_t l_row[4][kWaveRowList];
  __shared__ int32_t l_pos[4][kWaveRowList];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int bh = blockIdx.x * 4 + wv;
  if (bh >= BH) return;                                      // wave-uniform
  const uint64_t lt = (1ull << lane) - 1ull;
  const int Hq = A.Hq, Hkv = A.Hkv, P = A.P;
  const int b = bh / Hq, hq = bh % Hq, hkv = hq / (Hq / Hkv);
  const int lrow = A.grouped ? b * Hkv + hkv : bh;
  const T* v_pool = (const T*)A.v_pool;
  const float beta = A.beta; const int ibeta = A.ibeta;
  float* out = A.out + (size_t)bh * kD;
  const float* zr = A.zbuf + (size_t)bh * A.zstride;
  const int n_cand = min(clampi(A.n_sel[lrow], 0, A.cap) * P, 64 * KZ);
  const float seed_z = A.ex.tau_seed != nullptr ? A.ex.tau_seed[bh] : NAN;
  float u[KZ];
#pragma unroll
  for (int i = 0; i < KZ; ++i) u[i] = zr[min(i * 64 + lane, max(n_cand - 1, 0))];
  float zmax = -INFINITY;
#pragma unroll
  for (int i = 0; i < KZ; ++i) { u[i] = i * 64 + lane < n_cand ? u[i] : -INFINITY; zmax = fmaxf(zmax, u[i]); }
  zmax = wave_max(zmax);
  const bool want_kept = A.ex.tau_ref != nullptr && (A.ex.kept_mass_ref != nullptr || A.ex.kept_supp_ref != nullptr);
  if (!(zmax > -INFINITY)) {                                 // no valid candidate at all
    if (lane < 16) {
      *reinterpret_cast<float4*>(out + 8 * lane) = make_float4(0.f, 0.f, 0.f, 0.f);
      *reinterpret_cast<float4*>(out + 8 * lane + 4) = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    if (lane == 0) {
      A.tau_out[bh] = INFINITY; A.supp_out[bh] = 0;
      if (A.ex.solve_evals != nullptr) A.ex.solve_evals[bh] = 0;
      if (want_kept && A.ex.kept_mass_ref != nullptr) A.ex.kept_mass_ref[bh] = 0.f;
      if (want_kept && A.ex.kept_supp_ref != nullptr) A.ex.kept_supp_ref[bh] = 0;
    }
    return;
  }
  if (want_kept) {                                           // mass and count above a given threshold, all candidates
    const float tr = A.ex.tau_ref[bh];
    float f = 0.f; int c = 0;
#pragma unroll
    for (int i = 0; i < KZ; ++i) {
      const float x = u[i] - tr;
      if (x > 0.f) { f += pow_beta(x, beta, ibeta); ++c; }
    }
    f = wave_sum(f); c = wave_sum_i(c);
    if (lane == 0) {
      if (A.ex.kept_mass_ref != nullptr) A.ex.kept_mass_ref[bh] = f;
      if (A.ex.kept_supp_ref != nullptr) A.ex.kept_supp_ref[bh] = c;
    }
  }
#pragma unroll
  for (int i = 0; i < KZ; ++i) u[i] -= zmax;
  const float lo_u = -1.0f - 4e-6f * fmaxf(1.f, fabsf(zmax));
  int supp = 0, evals = 0;
  float tau_u;
  // Only candidates above zmax - 1 can be in the support: usually a few dozen.  They are compacted (in order)
  // into the LDS list and the threshold is solved over four registers per lane; if there are more than the list
  // holds, it is solved over all KZ registers.
  int n_c = 0;
#pragma unroll
  for (int i = 0; i < KZ; ++i) {
    const bool in = u[i] > lo_u;
    const uint64_t mk = __ballot(in);
    const int r = n_c + __popcll(mk & lt);
    if (in && r < kWaveRowList) { l_p[wv][r] = u[i]; l_pos[wv][r] = i * 64 + lane; }
    n_c += __popcll(mk);
  }
  const bool short_list = n_c <= kWaveRowList;               // wave-uniform
  float uu[kWaveRowList / 64]; int pp[kWaveRowList / 64];
  if (short_list) {
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int k = 0; k < kWaveRowList / 64; ++k) {
      const int e = lane + 64 * k;
      uu[k] = e < n_c ? l_p[wv][e] : -INFINITY;
      pp[k] = e < n_c ? l_pos[wv][e] : 0;
    }
    __builtin_amdgcn_wave_barrier();
    tau_u = solve_tau_regs(uu, lo_u, seed_z - zmax, beta, ibeta, supp, evals);
  } else {
    tau_u = solve_tau_core([&](float t, float& F, float& D, int& cnt) {
      float f = 0.f, d = 0.f; int c = 0;
#pragma unroll
      for (int i = 0; i < KZ; ++i) {
        const float x = u[i] - t;
        if (x > 0.f) { f += pow_beta(x, beta, ibeta); d += pow_beta_m1(x, beta, ibeta); ++c; }
      }
      F = wave_sum(f); D = beta * wave_sum(d); cnt = wave_sum_i(c);
    }, lo_u, seed_z - zmax, ibeta, supp, evals);
  }

  // weighted value sum: the support in candidate order through the LDS list; 4 row slots x 16 lanes gather it
  const int rs = lane >> 4, c = lane & 15;
  float acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) acc[i] = 0.f;
  int32_t* tok_dst = A.ex.support_tokens != nullptr ? A.ex.support_tokens + (size_t)bh * A.ex.support_cap : nullptr;
  // the support in candidate order, kWaveRowList tokens per pass (normally one pass): entry of rank r goes to
  // slot r - w0 of the list (the unrolled loop over the registers has no gather inside, so the code stays small)
  for (int w0 = 0; w0 < supp; w0 += kWaveRowList) {
    int run = 0;
    if (short_list) {                                        // one pass: the support is a subset of the list
#pragma unroll
      for (int k = 0; k < kWaveRowList / 64; ++k) {
        const float x = uu[k] - tau_u;
        const bool in = x > 0.f;
        const uint64_t mk = __ballot(in);
        const int r = run + __popcll(mk & lt);
        if (in) { l_p[wv][r] = pow_beta(x, beta, ibeta); l_pos[wv][r] = pp[k]; }
        run += __popcll(mk);
      }
    } else {
#pragma unroll
      for (int i = 0; i < KZ; ++i) {
        const float x = u[i] - tau_u;
        const bool in = x > 0.f;
        const uint64_t mk = __ballot(in);
        const int r = run + __popcll(mk & lt) - w0;
        if (in && r >= 0 && r < kWaveRowList) { l_p[wv][r] = pow_beta(x, beta, ibeta); l_pos[wv][r] = i * 64 + lane; }
        run += __popcll(mk);
      }
    }
    const int n_list = min(supp - w0, kWaveRowList);
    __builtin_amdgcn_wave_barrier();
    {
      // V rows of the listed tokens: page list -> block table, all lookups of the pass in flight together
      uint32_t rw[kWaveRowList / 64];
#pragma unroll
      for (int j = 0; j < kWaveRowList / 64; ++j)
        rw[j] = v_row_of<false>(A, b, lrow, hkv, l_pos[wv][min(lane + 64 * j, n_list - 1)]);
#pragma unroll
      for (int j = 0; j < kWaveRowList / 64; ++j)
        if (lane + 64 * j < n_list) l_row[wv][lane + 64 * j] = rw[j];
    }
    __builtin_amdgcn_wave_barrier();
    for (int e0 = 0; e0 < n_list; e0 += 32) {
      Raw8<T> vr[8]; float pw[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int e = e0 + 4 * j + rs;
        const int ec = min(e, n_list - 1);                   // clamped: loads stay unconditional
        pw[j] = e < n_list ? l_p[wv][ec] : 0.f;
        load_raw8(v_pool + (size_t)l_row[wv][ec] * kD + 8 * c, vr[j]);
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        float vv[8];
        widen8(vr[j], vv);
#pragma unroll
        for (int q = 0; q < 8; ++q) acc[q] = fmaf(pw[j], vv[q], acc[q]);
      }
    }
    if (tok_dst != nullptr) {
      for (int e = lane; e < n_list && w0 + e < A.ex.support_cap; e += 64)
        tok_dst[w0 + e] = token_of<false>(A, lrow, l_pos[wv][e]);
    }
    __builtin_amdgcn_wave_barrier();
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    acc[i] += __shfl_xor(acc[i], 16);
    acc[i] += __shfl_xor(acc[i], 32);
  }
  if (lane < 16) {
    *reinterpret_cast<float4*>(out + 8 * c) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    *reinterpret_cast<float4*>(out + 8 * c + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
  }
  if (lane == 0) {
    A.tau_out[bh] = tau_u + zmax; A.supp_out[bh] = supp;
    if (A.ex.solve_evals != nullptr) A.ex.solve_evals[bh] = evals;
  }
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
// Wavefronts of a pass-1 launch: enough to fill every compute unit several times over, never more than the
// lists can hold items; independent of how full the lists are.
static int device_compute_units() {
  static int cus[64] = {0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  if (cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
    cus[dev] = n;
  }
  return cus[dev];
}
// Workgroups per compute unit in a pass-1 launch.  Eight are resident at a time; launching twice that (when there
// is that much work) measured 3-5 % faster than a grid of resident workgroups only -- a wavefront that starts fresh
// streams better than one that loops -- while workgroups that find no work cost about half a microsecond per
// thousand, which bounds what a list capacity far above the lists' lengths can cost.  Every workgroup reads the U
// lengths, so launches with many units get fewer.
// When every page is a candidate the launch is large whatever the lists hold, and one item per wavefront, left to
// the hardware's scheduling, measured 2-3 % faster than eight per wavefront (five alternating pairs at 1M tokens:
// 417-459 against 431-467 us; 64 sequences of 8K tokens, 512 units: 222 against 237 us): such launches get up to
// 128 workgroups per compute unit (32 when the units are so many that reading their lengths is a cost of its own).
static int score_wgs_per_cu(int U, bool all_pages) {
  if (all_pages) return U <= 1024 ? 128 : 32;
  return U <= 256 ? 16 : 8;
}

template <int G, int MODE>
static void launch_scores(const Dims& dm, ScoreArgs sa, int32_t* pre_ws, hipStream_t st) {
  const int gp = pmax_pages(dm.P);
  const long long max_items = (long long)sa.U * (((MODE == kAllPages ? dm.Mmax : dm.cap) + gp - 1) / gp);
  long long wgs = (max_items + kScoreWaves - 1) / kScoreWaves;
  const long long wg_cap = (long long)device_compute_units() * score_wgs_per_cu(sa.U, MODE == kAllPages);
  if (wgs > wg_cap) wgs = wg_cap;
  if (wgs < 1) wgs = 1;
  dim3 grid((unsigned)wgs), block(kScoreThreads);
  const bool pre_global = sa.U > kUnitsLdsMax;
  const size_t lds = pre_global ? 0 : (size_t)(sa.U + 1) * sizeof(int);
  if (pre_global) {
    sa.pre_g = pre_ws;
    hipLaunchKernelGGL((unit_prefix_kernel<MODE>), dim3(1), dim3(1024), 0, st, sa, pre_ws);
  }
#define EKV_SCORES(KERNEL, ...)                                                                          \
  do {                                                                                                   \
    if (pre_global) hipLaunchKernelGGL((KERNEL<__VA_ARGS__, true>), grid, block, lds, st, sa);            \
    else hipLaunchKernelGGL((KERNEL<__VA_ARGS__, false>), grid, block, lds, st, sa);                      \
  } while (0)
  if (dm.dtype == EKV_BF16 && dm.P == 16) EKV_SCORES(decode_scores_mfma_kernel, G, MODE, 16);
  else if (dm.dtype == EKV_BF16 && dm.P == 32) EKV_SCORES(decode_scores_mfma_kernel, G, MODE, 32);
  else if (dm.dtype == EKV_BF16 && dm.P == 64) EKV_SCORES(decode_scores_mfma_kernel, G, MODE, 64);
  else if (dm.dtype == EKV_BF16) EKV_SCORES(decode_scores_valu_kernel, bf16_t, G, MODE);
  else EKV_SCORES(decode_scores_valu_kernel, float, G, MODE);
#undef EKV_SCORES
}

size_t decode_ws_carve(const Dims& dm, bool dense, void* base, DecodeWorkspace* ws) {
  const size_t slots = dense ? dm.Mmax : dm.cap;
  const size_t rows = (size_t)dm.B * dm.Hq;
  const size_t zstride = slots * dm.P;
  const int n_chunks_max = (int)((slots + pmax_pages(dm.P) - 1) / pmax_pages(dm.P));
  size_t n_slices = ((size_t)n_chunks_max + kFilterSliceChunks - 1) / kFilterSliceChunks;
  if (n_chunks_max <= kPreGroups || n_slices > (size_t)kFilterMaxSlices) n_slices = 0;
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += (bytes + 255) & ~(size_t)255; return o; };
  const size_t o_z = take(rows * zstride * sizeof(float));
  const size_t o_pm = take(rows * n_chunks_max * sizeof(float));
  const size_t o_pre = take((rows + 1) * sizeof(int32_t));
  // overflow list of a row whose candidates outgrow the solve's LDS list: (u, position) per entry
  const size_t spill_cap = zstride > (size_t)kListCap ? (zstride < (size_t)kSpillCap ? zstride : (size_t)kSpillCap) : 0;
  const size_t o_su = spill_cap ? take(rows * spill_cap * sizeof(float)) : 0;
  const size_t o_sp = spill_cap ? take(rows * spill_cap * sizeof(int32_t)) : 0;
  size_t o_fc = 0, o_fr = 0, o_fu = 0, o_fp = 0;
  if (n_slices) {
    o_fc = take(rows * n_slices * sizeof(int32_t));
    o_fr = take(rows * 2 * sizeof(float));
    o_fu = take(rows * n_slices * kFilterSliceCap * sizeof(float));
    o_fp = take(rows * n_slices * kFilterSliceCap * sizeof(int32_t));
  }
  if (ws != nullptr && base != nullptr) {
    char* p = (char*)base;
    ws->z = (float*)(p + o_z); ws->pmax = (float*)(p + o_pm); ws->unit_pre = (int32_t*)(p + o_pre);
    ws->zstride = zstride; ws->n_chunks_max = n_chunks_max; ws->n_slices_max = (int)n_slices;
    ws->spill_u = spill_cap ? (float*)(p + o_su) : nullptr;
    ws->spill_pos = spill_cap ? (int32_t*)(p + o_sp) : nullptr;
    ws->spill_cap = (int)spill_cap;
    ws->fcount = n_slices ? (int32_t*)(p + o_fc) : nullptr;
    ws->frow = n_slices ? (float*)(p + o_fr) : nullptr;
    ws->flist_u = n_slices ? (float*)(p + o_fu) : nullptr;
    ws->flist_pos = n_slices ? (int32_t*)(p + o_fp) : nullptr;
  }
  return off;
}

void launch_decode(const Dims& dm, bool dense, bool grouped, const void* q, const ekv_cache_view& c,
                   const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau, int32_t* supp,
                   const ekv_decode_extras& ex, const DecodeWorkspace& ws, hipStream_t st) {
  ScoreArgs sa{q, c.k_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws.z, ws.pmax,
               dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, ws.n_chunks_max, c.n_phys_pages, ws.zstride, dm.a * dm.scale,
               dm.HkvPool, 0, nullptr};
  SolveArgs so{c.v_pool, c.block_table, c.seq_lens, page_idx, n_sel, ws.z, ws.pmax, out, tau, supp, ex,
               dm.Hq, dm.Hkv, dm.P, dm.Mmax, dm.cap, ws.n_chunks_max, c.n_phys_pages, ws.zstride, dm.a, dm.beta, dm.ibeta};
  so.fcount = ws.fcount; so.frow = ws.frow; so.flist_u = ws.flist_u; so.flist_pos = ws.flist_pos;
  so.n_slices_max = ws.n_slices_max;
  so.grouped = grouped ? 1 : 0;
  so.HkvPool = dm.HkvPool;
  so.spill_u = ws.spill_u; so.spill_pos = ws.spill_pos; so.spill_cap = ws.spill_cap;
  FilterArgs fa{c.seq_lens, n_sel, ws.z, ws.pmax, ws.fcount, ws.frow, ws.flist_u, ws.flist_pos,
                dm.Hq, dm.Hkv, grouped ? 1 : 0, dm.P, ws.n_slices_max, dense ? dm.Mmax : dm.cap, ws.n_chunks_max,
                ws.zstride, dm.beta, dm.ibeta};
  dim3 fgrid(ws.n_slices_max, dm.B * dm.Hq), fblock(kFilterThreads);
  dim3 sgrid(dm.B * dm.Hq), sblock(kSolveThreads);
  if (dense) {
    sa.U = dm.B * dm.Hkv;
    switch (dm.G) {
      case 1: launch_scores<1, kAllPages>(dm, sa, ws.unit_pre, st); break;
      case 2: launch_scores<2, kAllPages>(dm, sa, ws.unit_pre, st); break;
      case 4: launch_scores<4, kAllPages>(dm, sa, ws.unit_pre, st); break;
      default: launch_scores<8, kAllPages>(dm, sa, ws.unit_pre, st); break;
    }
    if (ex.score_pass_only) return;
    if (ws.fcount != nullptr) {
      hipLaunchKernelGGL((filter_level_kernel<true>), dim3(dm.B * dm.Hq), fblock, 0, st, fa);
      hipLaunchKernelGGL((filter_compact_kernel<true>), fgrid, fblock, 0, st, fa);
    }
    if (dm.dtype == EKV_F32) hipLaunchKernelGGL((decode_solve_kernel<float, true>), sgrid, sblock, 0, st, so);
    else hipLaunchKernelGGL((decode_solve_kernel<bf16_t, true>), sgrid, sblock, 0, st, so);
  } else {
    if (grouped && dm.G > 1) {
      sa.U = dm.B * dm.Hkv;
      switch (dm.G) {
        case 2: launch_scores<2, kGroupList>(dm, sa, ws.unit_pre, st); break;
        case 4: launch_scores<4, kGroupList>(dm, sa, ws.unit_pre, st); break;
        default: launch_scores<8, kGroupList>(dm, sa, ws.unit_pre, st); break;
      }
    } else {                                    // G == 1: a group list is a per-head list
      sa.U = dm.B * dm.Hq;
      launch_scores<1, kPerHead>(dm, sa, ws.unit_pre, st);
    }
    if (ex.score_pass_only) return;
    if (ws.fcount != nullptr) {
      hipLaunchKernelGGL((filter_level_kernel<false>), dim3(dm.B * dm.Hq), fblock, 0, st, fa);
      hipLaunchKernelGGL((filter_compact_kernel<false>), fgrid, fblock, 0, st, fa);
    }
    const int rows = dm.B * dm.Hq;
    const long long max_cand = (long long)dm.cap * dm.P;
    if (ws.fcount == nullptr && max_cand <= 2048 && rows > kWaveRowsMin) {
      // many short rows: one wavefront per row
      dim3 wgrid((rows + 3) / 4), wblock(256);
      if (dm.dtype == EKV_F32) {
        if (max_cand <= 1024) hipLaunchKernelGGL((decode_solve_wave_kernel<float, 16>), wgrid, wblock, 0, st, so, rows);
        else hipLaunchKernelGGL((decode_solve_wave_kernel<float, 32>), wgrid, wblock, 0, st, so, rows);
      } else {
        if (max_cand <= 1024) hipLaunchKernelGGL((decode_solve_wave_kernel<bf16_t, 16>), wgrid, wblock, 0, st, so, rows);
        else hipLaunchKernelGGL((decode_solve_wave_kernel<bf16_t, 32>), wgrid, wblock, 0, st, so, rows);
      }
      return;
    }
    if (dm.dtype == EKV_F32) hipLaunchKernelGGL((decode_solve_kernel<float, false>), sgrid, sblock, 0, st, so);
    else hipLaunchKernelGGL((decode_solve_kernel<bf16_t, false>), sgrid, sblock, 0, st, so);
  }
}

}  // namespace ekv
