// Gaussian-aware entmax selector (paper Sec. 4.3 Eq. 10-12, App. D).
//
// Per (sequence, query head): solve  F(tau) = sum_p cnt_p * E[(a S_p - tau)_+^beta] = 1  for tau_hat,
// S_p ~ N(mu_p, sigma_p^2), with the truncated Gaussian moments in closed form (integer beta), then
// keep the pages whose estimated maximum a*(mu_p + sigma_p*z_cnt) exceeds tau_hat - margin and write
// them in ascending order.
//
// One evaluation of F costs an erfc and an exp per page, so the pages of a head are split over many
// workgroups.  The root iteration is a fixed sequence of launches without host involvement: launch k
// first advances the iteration state from the partial sums of launch k-1 (every workgroup repeats the
// same few scalar operations), then evaluates its slice at the new tau; once converged the remaining
// launches return at once.  A last kernel applies the selection rule.
//
// Root finding: F is positive, decreasing and convex.  The start is the root of the same equation for a
// single Gaussian with the pooled mean and variance of all pages; the iteration is Newton on log F
// kept inside a bracket [lo, hi] with F(lo) >= 1 > F(hi) (a step that leaves it is replaced by
// bisection).  The left end a*mu_max - 1 is valid because cnt*E[(Y)_+^beta] >= cnt*(E Y)_+^beta >= 1
// there (Jensen).
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

constexpr float kInvSqrt2 = 0.70710678118654752f;
constexpr float kInvSqrt2Pi = 0.39894228040143268f;
constexpr int kGaussEvalThreads = 256;
constexpr int kGaussMaxSplits = 64;
constexpr int kGaussIters = 8;            // evaluation launches per call (converged ones return at once)

// h_n(t) = E[(t + Z)_+^n], Z ~ N(0,1), for n = NB and NB-1 (so that M_n = sigma^n h_n).
// t >= -2.5: forward recurrence h_n = t h_{n-1} + (n-1) h_{n-2} from h_0 = Phi(t), h_1 = t Phi + phi.
// t <  -2.5: the forward recurrence cancels catastrophically; the same three-term recurrence run
// backwards from a high index (h_{n-2} = (h_n - t h_{n-1})/(n-1), all terms positive) and normalised
// by h_0 = Phi(t) is stable there (Miller's algorithm).
template <int NB>
__device__ __forceinline__ void trunc_h(float t, float& h_nb, float& h_nbm1) {
  if (t < -13.f) { h_nb = 0.f; h_nbm1 = 0.f; return; }      // below float32 resolution of the sum
  const float Phi = 0.5f * erfcf(-t * kInvSqrt2);
  if (t >= -2.5f) {
    const float phi = expf(-0.5f * t * t) * kInvSqrt2Pi;
    float h[5];
    h[0] = Phi;
    h[1] = fmaf(t, Phi, phi);
#pragma unroll
    for (int n = 2; n <= NB; ++n) h[n] = fmaf(t, h[n - 1], (float)(n - 1) * h[n - 2]);
    h_nb = h[NB]; h_nbm1 = h[NB - 1];
  } else {
    constexpr int N = 26;
    float hn1 = 0.f, hn = 1.f;            // h_{n}, h_{n-1} at n = N + 1
    float cap_nb = 0.f, cap_nbm1 = 0.f;
#pragma unroll
    for (int n = N + 1; n >= 2; --n) {
      const float hm = (hn1 - t * hn) * (1.0f / (float)(n - 1));    // h_{n-2}
      hn1 = hn; hn = hm;
      if (n - 2 == NB) cap_nb = hn;
      if (n - 2 == NB - 1) cap_nbm1 = hn;
    }
    const float s = Phi / hn;             // hn = unnormalised h_0
    h_nb = cap_nb * s; h_nbm1 = cap_nbm1 * s;
  }
}

// cnt * M_NB and cnt * M_{NB-1} of Y ~ N(muY, sY^2)
template <int NB>
__device__ __forceinline__ void page_mass(float muY, float sY, float cnt, float& f, float& d) {
  if (sY > 1e-30f) {
    float hb, hbm1;
    trunc_h<NB>(muY / sY, hb, hbm1);
    float sp = 1.f;                        // sY^(NB-1)
#pragma unroll
    for (int i = 0; i < NB - 1; ++i) sp *= sY;
    f = cnt * sp * sY * hb;
    d = cnt * sp * hbm1;
  } else {
    const float m = fmaxf(muY, 0.f);
    float mp = 1.f;
#pragma unroll
    for (int i = 0; i < NB - 1; ++i) mp *= m;
    f = cnt * mp * m;
    d = (NB == 1) ? (muY > 0.f ? cnt : 0.f) : cnt * mp;
  }
}

// Iteration state of one (b,h): the point the next evaluation is taken at, and its bracket.
struct GaussState { float tau, lo, hi; int done; };

// workspace: state[2][BH], init partials [BH][S][4], eval partials [2][BH][S][2]
struct GaussWs {
  GaussState* state; float* init_part; float* eval_part; int S;
};

__device__ __forceinline__ float bcast_wave0_sum(float v, float* slot) {
  // sum over the lanes of wavefront 0 (fixed order), broadcast to the block
  v = wave_sum(v);
  __syncthreads();
  if (threadIdx.x == 0) *slot = v;
  __syncthreads();
  return *slot;
}

// Launch 0 of a call: slice partials of max a*mu and of the pooled first and second moments.
__global__ __launch_bounds__(kGaussEvalThreads) void gauss_init_kernel(const float* __restrict__ mu,
                                                                       const float* __restrict__ sigma,
                                                                       const int32_t* __restrict__ seq_lens,
                                                                       GaussWs ws, float a, int Hq, int P, int Mmax) {
  __shared__ float red[kGaussEvalThreads / 64][4];
  const int bh = blockIdx.y, s = blockIdx.x, b = bh / Hq, tid = threadIdx.x;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const float cnt_last = (float)(n - (M - 1) * P);
  const int per = (M + ws.S - 1) / ws.S;
  const int p0 = s * per, p1 = min(p0 + per, M);
  float mx = -INFINITY, s0 = 0.f, s1 = 0.f, s2 = 0.f;
  for (int p = p0 + tid; p < p1; p += kGaussEvalThreads) {
    const float m = a * mu[(size_t)bh * Mmax + p], sd = a * sigma[(size_t)bh * Mmax + p];
    const float c = p == M - 1 ? cnt_last : (float)P;
    mx = fmaxf(mx, m); s0 += c; s1 = fmaf(c, m, s1); s2 = fmaf(c, fmaf(m, m, sd * sd), s2);
  }
  mx = wave_max(mx); s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2);
  if ((tid & 63) == 0) { red[tid >> 6][0] = mx; red[tid >> 6][1] = s0; red[tid >> 6][2] = s1; red[tid >> 6][3] = s2; }
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < kGaussEvalThreads / 64; ++i) {
      mx = fmaxf(mx, red[i][0]); s0 += red[i][1]; s1 += red[i][2]; s2 += red[i][3];
    }
    float* o = ws.init_part + ((size_t)bh * ws.S + s) * 4;
    o[0] = mx; o[1] = s0; o[2] = s1; o[3] = s2;
  }
}

// Scalar solve of n * sd^NB * h_NB((m - tau)/sd) = 1 (the pooled single-Gaussian model), started at `lo`.
template <int NB>
__device__ float pooled_guess(float n, float m, float sd, float lo) {
  float tau = lo, hi = INFINITY, l = lo;
  for (int it = 0; it < 24; ++it) {
    float f, d;
    page_mass<NB>(m - tau, sd, n, f, d);
    d *= (float)NB;
    if (f >= 1.f) l = tau; else hi = tau;
    float next = (f > 0.f && d > 0.f) ? tau + f * __logf(f) / d : 0.5f * (l + tau);
    if (hi < INFINITY && !(next > l && next < hi)) next = 0.5f * (l + hi);
    if (fabsf(next - tau) <= 1e-4f) { tau = next; break; }
    tau = next;
  }
  return fmaxf(tau, lo);
}

// Advance the iteration state with the result (F, D = -dF/dtau) of the evaluation at st.tau.
__device__ __forceinline__ GaussState advance_state(GaussState st, float F, float D) {
  if (st.done) return st;
  if (fabsf(F - 1.0f) <= 2e-6f) { st.done = 1; return st; }         // float32 resolution of F: tau is the root
  if (F >= 1.0f) st.lo = st.tau; else st.hi = st.tau;
  float next = st.tau;
  bool ok = false;
  if (F > 0.f && D > 0.f) {
    next = st.tau + F * __logf(F) / D;                              // Newton on log F
    ok = next > st.lo && next < st.hi;
    if (!ok) { next = st.tau + (F - 1.0f) / D; ok = next > st.lo && next < st.hi; }   // Newton on F
  }
  if (!ok) next = st.hi < INFINITY ? 0.5f * (st.lo + st.hi) : st.lo + 1.0f;
  if (fabsf(next - st.tau) <= 3e-7f * fmaxf(1.f, fabsf(next))) st.done = 1;
  st.tau = next;
  return st;
}

template <int NB>
__global__ __launch_bounds__(kGaussEvalThreads) void gauss_eval_kernel(const float* __restrict__ mu,
                                                                       const float* __restrict__ sigma,
                                                                       const int32_t* __restrict__ seq_lens,
                                                                       GaussWs ws, int k, float a, int Hq, int P,
                                                                       int Mmax, int BH) {
  __shared__ float red[kGaussEvalThreads / 64][2];
  __shared__ float bc[4];
  const int bh = blockIdx.y, s = blockIdx.x, b = bh / Hq, tid = threadIdx.x;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const float cnt_last = (float)(n - (M - 1) * P);
  GaussState st;
  if (k == 0) {
    // start: left end from max a*mu, first point from the pooled single-Gaussian model
    float mx = -INFINITY, s0 = 0.f, s1 = 0.f, s2 = 0.f;
    if (tid < ws.S) {
      const float* o = ws.init_part + ((size_t)bh * ws.S + tid) * 4;
      mx = o[0]; s0 = o[1]; s1 = o[2]; s2 = o[3];
    }
    if (tid < 64) { mx = wave_max(mx); s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2); }
    if (tid == 0) { bc[0] = mx; bc[1] = s0; bc[2] = s1; bc[3] = s2; }
    __syncthreads();
    mx = bc[0]; s0 = bc[1]; s1 = bc[2]; s2 = bc[3];
    const float mean = s1 / s0;
    const float var = fmaxf(s2 / s0 - mean * mean, 0.f);
    st.lo = mx - 1.0f; st.hi = INFINITY; st.done = 0;
    st.tau = pooled_guess<NB>(s0, mean, sqrtf(var), st.lo);
  } else {
    st = ws.state[(size_t)((k - 1) & 1) * BH + bh];
    float F = 0.f, D = 0.f;
    if (tid < ws.S) {
      const float* o = ws.eval_part + (((size_t)((k - 1) & 1) * BH + bh) * ws.S + tid) * 2;
      F = o[0]; D = o[1];
    }
    if (tid < 64) { F = wave_sum(F); D = wave_sum(D); }
    if (tid == 0) { bc[0] = F; bc[1] = D; }
    __syncthreads();
    st = advance_state(st, bc[0], (float)NB * bc[1]);
  }
  if (s == 0 && tid == 0) ws.state[(size_t)(k & 1) * BH + bh] = st;
  if (st.done) return;

  const int per = (M + ws.S - 1) / ws.S;
  const int p0 = s * per, p1 = min(p0 + per, M);
  float f = 0.f, d = 0.f;
  for (int p = p0 + tid; p < p1; p += kGaussEvalThreads) {
    float fp, dp;
    page_mass<NB>(fmaf(a, mu[(size_t)bh * Mmax + p], -st.tau), a * sigma[(size_t)bh * Mmax + p],
                  p == M - 1 ? cnt_last : (float)P, fp, dp);
    f += fp; d += dp;
  }
  f = wave_sum(f); d = wave_sum(d);
  if ((tid & 63) == 0) { red[tid >> 6][0] = f; red[tid >> 6][1] = d; }
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < kGaussEvalThreads / 64; ++i) { f += red[i][0]; d += red[i][1]; }
    float* o = ws.eval_part + (((size_t)(k & 1) * BH + bh) * ws.S + s) * 2;
    o[0] = f; o[1] = d;
  }
}

struct ZqTable { float z[65]; };   // z[c] = PhiInv(q_page^(1/c)), c = 1..64

template <int NB, int ITEMS>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void gauss_select_kernel(
    const float* __restrict__ mu, const float* __restrict__ sigma, const int32_t* __restrict__ seq_lens,
    GaussWs ws, ZqTable zq, float margin, float a, float* __restrict__ tau_hat, int32_t* __restrict__ page_idx,
    int32_t* __restrict__ n_sel, int32_t* __restrict__ overflow, int Hq, int P, int Mmax, int cap, int BH) {
  __shared__ SelectShared sh;
  __shared__ float bc[2];
  const int bh = blockIdx.x, b = bh / Hq, tid = threadIdx.x;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  if (M <= 0) { if (tid == 0) { n_sel[bh] = 0; overflow[bh] = 0; tau_hat[bh] = 0.f; } return; }
  const int cnt_last = n - (M - 1) * P;
  const float* mu_r = mu + (size_t)bh * Mmax;
  const float* sg_r = sigma + (size_t)bh * Mmax;

  // last state update (the evaluation of launch kGaussIters-1)
  constexpr int kl = kGaussIters - 1;
  GaussState st = ws.state[(size_t)(kl & 1) * BH + bh];
  float F = 0.f, D = 0.f;
  if (tid < ws.S) {
    const float* o = ws.eval_part + (((size_t)(kl & 1) * BH + bh) * ws.S + tid) * 2;
    F = o[0]; D = o[1];
  }
  if (tid < 64) { F = wave_sum(F); D = wave_sum(D); }
  if (tid == 0) { bc[0] = F; bc[1] = D; }
  __syncthreads();
  st = advance_state(st, bc[0], (float)NB * bc[1]);
  const float tau = st.tau;
  if (tid == 0) tau_hat[bh] = tau;

  // selection: keep p iff a*(mu_p + sigma_p z_cnt) > tau - margin
  const float thr = tau - margin;
  const float z_full = zq.z[P], z_last = zq.z[cnt_last];
  auto keyfn = [=](int p) { return float_to_key(a * fmaf(sg_r[p], p == M - 1 ? z_last : z_full, mu_r[p])); };
  KeySet<ITEMS, decltype(keyfn)> ks(keyfn, M);
  const uint32_t kthr = float_to_key(thr);      // > 0, so empty slots (key 0) never pass
  int c = 0;
#pragma unroll
  for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) c += ks.key(i) > kthr;
  const int count = block_sum_i(c, sh.scan_buf);
  int32_t* out = page_idx + (size_t)bh * cap;
  int n_out, ovf = 0;
  if (count >= 1 && count <= cap) {
    compact_ordered(ks, kthr, 0, sh, out);
    n_out = count;
  } else {
    // nothing passed: the single best page; too many: the cap best pages (lower index on ties)
    const int k = count == 0 ? 1 : cap;
    ovf = count > cap;
    uint32_t vT; int k_eq;
    radix_select_kth(ks, k, sh, vT, k_eq);
    compact_ordered(ks, vT, k_eq, sh, out);
    n_out = k;
  }
  if (tid == 0) { n_sel[bh] = n_out; overflow[bh] = ovf; }
}

static int gauss_splits(const Dims& dm) {
  const int BH = dm.B * dm.Hq;
  int S = (4096 + BH - 1) / BH;
  const int max_by_pages = (dm.Mmax + kGaussEvalThreads - 1) / kGaussEvalThreads;   // >= 256 pages per slice
  if (S > max_by_pages) S = max_by_pages;
  if (S > kGaussMaxSplits) S = kGaussMaxSplits;
  if (S < 1) S = 1;
  return S;
}

size_t select_gauss_ws_bytes(const Dims& dm) {
  const size_t BH = (size_t)dm.B * dm.Hq, S = gauss_splits(dm);
  size_t b = 2 * BH * sizeof(GaussState) + BH * S * 4 * sizeof(float) + 2 * BH * S * 2 * sizeof(float);
  return (b + 255) & ~(size_t)255;
}

template <int NB>
static void launch_gauss_NB(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                            const ZqTable& zq, float margin, float* tau_hat, int32_t* page_idx, int32_t* n_sel,
                            int32_t* overflow, const GaussWs& ws, hipStream_t st) {
  const int BH = dm.B * dm.Hq;
  dim3 egrid(ws.S, BH), eblock(kGaussEvalThreads);
  hipLaunchKernelGGL(gauss_init_kernel, egrid, eblock, 0, st, mu, sigma, seq_lens, ws, dm.a, dm.Hq, dm.P, dm.Mmax);
  for (int k = 0; k < kGaussIters; ++k)
    hipLaunchKernelGGL(gauss_eval_kernel<NB>, egrid, eblock, 0, st, mu, sigma, seq_lens, ws, k, dm.a, dm.Hq, dm.P,
                       dm.Mmax, BH);
  dim3 sgrid(BH), sblock(kSelThreads);
#define EKV_GSEL(ITEMS)                                                                                         \
  hipLaunchKernelGGL((gauss_select_kernel<NB, ITEMS>), sgrid, sblock, 0, st, mu, sigma, seq_lens, ws, zq, margin, \
                     dm.a, tau_hat, page_idx, n_sel, overflow, dm.Hq, dm.P, dm.Mmax, dm.cap, BH)
  if (dm.Mmax <= 4 * kSelThreads) EKV_GSEL(4);
  else if (dm.Mmax <= 16 * kSelThreads) EKV_GSEL(16);
  else if (dm.Mmax <= 64 * kSelThreads) EKV_GSEL(64);
  else EKV_GSEL(0);
#undef EKV_GSEL
}

void launch_select_gauss(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                         const float* zq_table, float margin, float* tau_hat, int32_t* page_idx,
                         int32_t* n_sel, int32_t* overflow, void* workspace, hipStream_t st) {
  ZqTable zq;
  for (int i = 0; i < 65; ++i) zq.z[i] = zq_table[i];
  const size_t BH = (size_t)dm.B * dm.Hq;
  GaussWs ws;
  ws.S = gauss_splits(dm);
  ws.state = (GaussState*)workspace;
  ws.init_part = (float*)(ws.state + 2 * BH);
  ws.eval_part = ws.init_part + BH * ws.S * 4;
  switch (dm.ibeta) {
    case 1: launch_gauss_NB<1>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    case 2: launch_gauss_NB<2>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    case 3: launch_gauss_NB<3>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    default: launch_gauss_NB<4>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
  }
}

}  // namespace ekv
