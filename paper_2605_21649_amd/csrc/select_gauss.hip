// Gaussian-aware entmax selector (paper Sec. 4.3 Eq. 10-12, App. D).
//
// Per (sequence, query head): solve  F(tau) = sum_p cnt_p * E[(a S_p - tau)_+^beta] = 1  for tau_hat,
// S_p ~ N(mu_p, sigma_p^2), with the truncated Gaussian moments in closed form (integer beta), then
// keep the pages whose estimated maximum a*(mu_p + sigma_p*z_cnt) exceeds tau_hat - margin and write
// them in ascending order.
//
// One evaluation of F costs an exp and two short polynomials per page, so the pages of a head are split
// over many workgroups.  The root iteration is a fixed sequence of launches without host involvement:
// launch k first advances the iteration state from the partial sums of launch k-1 (every workgroup
// repeats the same few scalar operations), then evaluates its slice at the new tau.  The last evaluation
// launch also applies the selection rule SPECULATIVELY, at a threshold slightly below the one its own point
// implies: every wavefront writes the passing pages of its range, in order, with their estimates.  The final
// kernel takes the last state update, keeps the candidates above the final threshold and concatenates them
// in order; if the final threshold fell below the speculative one, or the iteration has not converged, its
// workgroup finishes the head alone over all pages (rare).
//
// Root finding: F is positive, decreasing and convex.  The start is the root of the same equation for a
// single Gaussian with the pooled mean and variance of all pages, raised to the root of the mixture of the
// hottest page of every wavefront of the first pass when that is higher (a few pages far above the bulk);
// the iteration is Halley's on log F kept inside a bracket [lo, hi] with F(lo) >= 1 > F(hi) (a step that
// leaves it falls back to Newton on log F, on F, then to bisection).  The left end a*mu_max - 1 is valid
// because cnt*E[(Y)_+^beta] >= cnt*(E Y)_+^beta >= 1 there (Jensen).
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

#include "trunc_tail_coeffs.inc"

constexpr float kInvSqrt2 = 0.70710678118654752f;
constexpr float kInvSqrt2Pi = 0.39894228040143268f;
constexpr int kGaussEvalThreads = 256;
constexpr int kGaussMaxSplits = 64;
// Evaluation launches per call.  The pooled start is within ~1e-2 of the root on the benchmark workloads, the
// first Newton step brings that to ~1e-5 and the second to ~1e-10, which advance_state recognises from the two
// step sizes without a third evaluation.  A launch that finds its head converged still costs 4.6 us (2048
// workgroups read the state and leave), about what the rare continuation inside the gather kernel costs, so
// there are no spare ones.
constexpr int kGaussIters = 2;
constexpr int kGaussSinglePages = 8192;    // heads of at most this many pages, in launches of at most ...
constexpr int kGaussSingleRows = 512;      // ... this many heads, are selected by one launch
constexpr int kGaussWaves = kGaussEvalThreads / 64;

template <int IV, int N>
__device__ __forceinline__ float horner_tail(float s) {
  float acc = kTailCoef[IV][N][kTailDeg];
#pragma unroll
  for (int k = kTailDeg - 1; k >= 0; --k) acc = fmaf(acc, s, kTailCoef[IV][N][k]);
  return acc;
}

// h_n(t) = E[(t + Z)_+^n], Z ~ N(0,1), for n = NB and NB-1 (so that M_n = sigma^n h_n).
// t >= -2.5: forward recurrence h_n = t h_{n-1} + (n-1) h_{n-2} from h_0 = Phi(t), h_1 = t Phi + phi
//            (the closed forms the paper prints for n = 1, 2, 3).
// t <  -2.5: those forms cancel catastrophically in float32; there h_n(t) = phi(t) * |t|^-(n+1) * P_n(1/t^2)
//            with fitted degree-8 polynomials (relative error 2e-7, see gen_trunc_tail_coeffs.py).
template <int NB>
__device__ __forceinline__ void trunc_h(float t, float& h_nb, float& h_nbm1, float& h_nbm2) {
  // h_nbm2 = h_{NB-2} (for the second derivative of F); for NB = 1 it is the density phi(t) = dPhi/dt
  if (t < -kTailXHi) { h_nb = 0.f; h_nbm1 = 0.f; h_nbm2 = 0.f; return; }   // below float32 resolution of the sum
  const float phi = __expf(-0.5f * t * t) * kInvSqrt2Pi;
  if (t >= -kTailXLo) {
    const float Phi = 0.5f * erfcf(-t * kInvSqrt2);
    float h[5];
    h[0] = Phi;
    h[1] = fmaf(t, Phi, phi);
#pragma unroll
    for (int n = 2; n <= NB; ++n) h[n] = fmaf(t, h[n - 1], (float)(n - 1) * h[n - 2]);
    h_nb = h[NB]; h_nbm1 = h[NB - 1]; h_nbm2 = NB >= 2 ? h[NB >= 2 ? NB - 2 : 0] : phi;
  } else {
    const float inv = __builtin_amdgcn_rcpf(-t), u = inv * inv;
    float p_nb, p_m1, p_m2 = 1.f;
    if (-t < kTailXSplit) {
      const float s = (u - kTailMid[0]) * kTailInvHalf[0];
      p_nb = horner_tail<0, NB>(s); p_m1 = horner_tail<0, NB - 1>(s);
      if (NB >= 2) p_m2 = horner_tail<0, (NB >= 2 ? NB - 2 : 0)>(s);
    } else {
      const float s = (u - kTailMid[1]) * kTailInvHalf[1];
      p_nb = horner_tail<1, NB>(s); p_m1 = horner_tail<1, NB - 1>(s);
      if (NB >= 2) p_m2 = horner_tail<1, (NB >= 2 ? NB - 2 : 0)>(s);
    }
    float ipm = phi;                       // phi * x^-(NB-1)
#pragma unroll
    for (int i = 0; i < NB - 1; ++i) ipm *= inv;
    const float ip = ipm * inv;            // phi * x^-NB
    h_nbm2 = NB >= 2 ? ipm * p_m2 : phi;
    h_nbm1 = ip * p_m1;
    h_nb = ip * inv * p_nb;
  }
}

// cnt * M_NB and cnt * M_{NB-1} of Y ~ N(muY, sY^2)
// Also d2 with F'' = NB * sum d2:  (NB-1) * cnt * M_{NB-2} for NB >= 2, cnt * density of Y at 0 for NB = 1.
template <int NB>
__device__ __forceinline__ void page_mass(float muY, float sY, float cnt, float& f, float& d, float& d2) {
  if (sY > 1e-30f) {
    float hb, hbm1, hbm2;
    const float rs = __builtin_amdgcn_rcpf(sY);
    trunc_h<NB>(muY * rs, hb, hbm1, hbm2);
    float sp2 = 1.f;                       // sY^(NB-2) (NB >= 2)
#pragma unroll
    for (int i = 0; i < NB - 2; ++i) sp2 *= sY;
    const float sp = NB >= 2 ? sp2 * sY : 1.f;     // sY^(NB-1)
    f = cnt * sp * sY * hb;
    d = cnt * sp * hbm1;
    d2 = NB >= 2 ? (float)(NB - 1) * cnt * sp2 * hbm2 : cnt * hbm2 * rs;
  } else {
    const float m = fmaxf(muY, 0.f);
    float mp2 = 1.f;                       // m^(NB-2) (NB >= 3)
#pragma unroll
    for (int i = 0; i < NB - 2; ++i) mp2 *= m;
    const float mp = NB >= 2 ? mp2 * m : 1.f;
    f = cnt * mp * m;
    d = (NB == 1) ? (muY > 0.f ? cnt : 0.f) : cnt * mp;
    d2 = NB >= 3 ? (float)(NB - 1) * cnt * mp2 : (NB == 2 && muY > 0.f ? cnt : 0.f);
  }
}
template <int NB>
__device__ __forceinline__ void page_mass(float muY, float sY, float cnt, float& f, float& d) {
  float d2;
  page_mass<NB>(muY, sY, cnt, f, d, d2);
}

// Iteration state of one (b,h): the point the next evaluation is taken at, and its bracket.
// `step` is the step that led to tau and `order` the order of the update that produced it (3: a Halley-type step,
// 2: Newton on log F, 0: none yet, or the point came from a fallback).
struct GaussState { float tau, lo, hi; int done; float step; int order; };

// workspace: state[2][BH], init partials [BH][S][4], eval partials [2][BH][S][3],
//            hottest page (a mu, a sigma, count) of every wavefront of the init launch [BH][S*4][3],
//            per wavefront of the last evaluation launch: count [BH][S*4] and candidate lists
//            (page, estimate) [BH][S*4][pw]
struct GaussWs {
  GaussState* state; float* init_part; float* eval_part; float* hot_part; int32_t* sel_cnt; int32_t* sel_page;
  float* sel_key;
  int S, per, pw;    // slices per head, pages per slice, pages per wavefront of a slice
};

struct ZqTable { float z[65]; };   // z[c] = PhiInv(q_page^(1/c)), c = 1..64

// The speculative selection threshold of an evaluation at tau: candidates are complete whenever the final
// threshold tau_hat - margin is not below it.
__device__ __forceinline__ float spec_threshold(float tau, float margin) {
  return tau - margin - 4e-3f * fmaxf(1.f, fabsf(tau));
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
  float hk = -INFINITY, hm = 0.f, hs = 1.f, hc = 0.f;      // this thread's hottest page: a(mu + 2 sigma) largest
  for (int p = p0 + tid; p < p1; p += kGaussEvalThreads) {
    const float m = a * mu[(size_t)bh * Mmax + p], sd = a * sigma[(size_t)bh * Mmax + p];
    const float c = p == M - 1 ? cnt_last : (float)P;
    mx = fmaxf(mx, m); s0 += c; s1 = fmaf(c, m, s1); s2 = fmaf(c, fmaf(m, m, sd * sd), s2);
    const float key = fmaf(2.f, sd, m);
    if (key > hk) { hk = key; hm = m; hs = sd; hc = c; }
  }
  {
    // the wavefront's hottest page (lowest lane on ties): one component of the start's mixture
    const float kmax = wave_max(hk);
    const uint64_t who = __ballot(hc > 0.f && hk == kmax);
    const int src = who ? __builtin_ctzll(who) : 0;
    const float wm = __shfl(hm, src), wsd = __shfl(hs, src), wc = who ? __shfl(hc, src) : 0.f;
    if ((tid & 63) == 0) {
      float* o = ws.hot_part + (((size_t)bh * ws.S + s) * kGaussWaves + (tid >> 6)) * 3;
      o[0] = wm; o[1] = wsd; o[2] = wc;
    }
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

// The single pooled Gaussian is a poor model when the page moments change along the sequence (a relevant segment,
// a recency trend, two populations one after the other): its variance then holds the spread BETWEEN the parts and
// its root can lie more than 1 above tau_hat, too far for the two evaluation launches.  The init launch already
// leaves the pooled moments of every slice of the sequence; the mixture of those (one Gaussian per slice, one slice
// per lane) follows such structure at the cost of the scalar iteration it replaces: Newton on log F_mix from the
// pooled model's leading-order tail estimate, kept inside the bracket the signs of log F_mix give (secant, then
// bisection towards `lo`, when a step leaves it).  On homogeneous pages the slices repeat the pooled moments and
// the root is the pooled one.  `n, m, sd`: this lane's slice (n = 0: none); `pn, pm, psd`: the pooled moments.
template <int NB>
__device__ __forceinline__ float slice_mixture_guess(float n, float m, float sd, float pn, float pm, float psd, float lo) {
  if (!(psd > 1e-20f)) return lo;
  float sp = pn;
#pragma unroll
  for (int i = 0; i < NB; ++i) sp *= psd;
  float tau = sp > 1.f ? pm + psd * sqrtf(2.f * __logf(sp)) : lo;
  tau = fmaxf(tau, lo);
  float blo = lo, bhi = INFINITY, glo = 0.f, ghi = 0.f, prev = 0.f;
  for (int it = 0; it < 12; ++it) {
    float f = 0.f, d = 0.f;
    if (n > 0.f) page_mass<NB>(m - tau, sd, n, f, d);
    f = wave_sum(f); d = (float)NB * wave_sum(d);            // wave-uniform from here on
    float next;
    bool newton = false;
    if (f > 0.f && d > 0.f) {
      const float g = __logf(f);
      if (g > 0.f) { blo = tau; glo = g; } else { bhi = tau; ghi = g; }
      next = fmaxf(tau + f * g / d, lo);                     // a step below the left end goes to the left end
      newton = next >= blo && next < bhi;
      if (!newton) next = bhi < INFINITY && glo > 0.f ? blo + (bhi - blo) * glo / (glo - ghi) : 0.5f * (blo + fminf(bhi, tau));
    } else {
      bhi = tau; ghi = -80.f;                                // nothing of the mixture reaches tau: go down
      next = 0.5f * (blo + tau);
    }
    next = fmaxf(next, lo);
    const float step = fabsf(next - tau);
    const bool close = step <= 1e-2f * psd ||
                       (newton && prev != 0.f && step <= 0.25f * prev && step * step * step <= 2e-2f * psd * prev * prev);
    tau = next;
    prev = newton ? step : 0.f;
    if (close) break;
  }
  return tau;
}

// The pooled model misses a few pages far above the bulk (their mass decides tau when they exist).  The hottest
// page of every wavefront of the init launch (at most 256 pages, four per lane here) gives F_hot <= F, so the
// root of F_hot = 1 is a lower bound of tau_hat: if F_hot(tau) > 1 at the pooled start, the start is moved to
// that root (Newton on log F_hot inside a bracket, secant on log F_hot when a step leaves it; to 2e-3 in
// log F_hot).  One wavefront; on homogeneous pages the first evaluation gives F_hot <= 1 and nothing changes.
struct HotPages { float m[4], s[4], c[4]; };

__device__ __forceinline__ HotPages load_hot_pages(const float* __restrict__ hot, int n_hot) {
  HotPages h;
  const int lane = threadIdx.x & 63;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = lane + 64 * j;
    const bool ok = i < n_hot;
    const float* o = hot + (size_t)(ok ? i : 0) * 3;
    h.m[j] = o[0]; h.s[j] = o[1]; h.c[j] = ok ? o[2] : 0.f;
  }
  return h;
}

template <int NB>
__device__ __forceinline__ float raise_to_hot_pages(float tau, const HotPages& h) {
  float lo = -INFINITY, hi = INFINITY, glo = 0.f, ghi = 0.f;
  for (int it = 0; it < 10; ++it) {
    float f = 0.f, d = 0.f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (h.c[j] > 0.f) {
        float fp, dp;
        page_mass<NB>(h.m[j] - tau, h.s[j], h.c[j], fp, dp);
        f += fp; d += dp;
      }
    }
    f = wave_sum(f); d = (float)NB * wave_sum(d);          // wave-uniform from here on
    if (it == 0 && !(f > 1.0f)) break;                     // the pooled start is not below the hot pages' root
    if (!(f > 0.f && d > 0.f)) { if (lo > -INFINITY) tau = lo; break; }
    const float g = __logf(f);
    if (fabsf(g) <= 2e-2f) break;
    if (g > 0.f) { lo = tau; glo = g; } else { hi = tau; ghi = g; }
    float next = tau + f * g / d;
    if (!(next > lo && next < hi)) next = lo + (hi - lo) * glo / (glo - ghi);
    tau = next;
  }
  return tau;
}

// Advance the iteration state with the result (F, D = -dF/dtau, D2 = d2F/dtau2) of the evaluation at st.tau.
// The update works on g = log F, which is close to a parabola wherever Gaussian tails make up F: the step is the
// root of g's local quadratic model nearest to Newton's (Halley's method in its irrational form; the paper names
// Newton or Halley, and the third moment this needs comes with the other two), then Halley's rational step,
// then Newton's on log F and on F, then bisection, whichever first stays inside the bracket.  A start 2.8 above
// the root of a two-population mixture comes within 3e-2 in one such step and 4e-8 in two (float64 simulation;
// the rational form: 8e-2, 3e-6).
// Stopping: F = 1 to float32 resolution; or a step below the resolution of tau; or two consecutive smooth steps
// s1, s2 with |s2| <= |s1|/20 whose implied remaining error is below 1e-7 (relative to max(1, |tau|)) without
// evaluating F at the new point: an iteration of order 2 shrinks the error as e' = K e^2 with K = |s2|/s1^2, so
// after the second step it is about |s2|^3/s1^2; when both steps are third-order ones, e' = K e^3 with
// K = |s2|/|s1|^3 and the remaining error is about s2^4/|s1|^3, taken with a factor 10.
__device__ __forceinline__ GaussState advance_state(GaussState st, float F, float D, float D2) {
  if (st.done) return st;
  if (fabsf(F - 1.0f) <= 2e-6f) { st.done = 1; return st; }         // float32 resolution of F: tau is the root
  if (F >= 1.0f) st.lo = st.tau; else st.hi = st.tau;
  float next = st.tau;
  bool ok = false;
  int order = 0;
  if (F > 0.f && D > 0.f) {
    // g = log F:  g' = -D/F < 0,  g'' = D2/F - (D/F)^2
    const float g = __logf(F), g1 = -D / F, g2 = D2 / F - g1 * g1;
    const float disc = g1 * g1 - 2.f * g * g2;
    if (disc > 0.f) {                                               // g + g' d + g'' d^2 / 2 = 0, the root next to -g/g'
      next = st.tau - 2.f * g / (g1 - sqrtf(disc));
      ok = next > st.lo && next < st.hi;
    }
    if (!ok) {                                                      // Halley: -2 g g' / (2 g'^2 - g g'')
      const float den = 2.f * g1 * g1 - g * g2;
      if (den > 0.f) { next = st.tau - 2.f * g * g1 / den; ok = next > st.lo && next < st.hi; }
    }
    if (ok) order = 3;
    if (!ok) { next = st.tau - g / g1; ok = next > st.lo && next < st.hi; if (ok) order = 2; }   // Newton on log F
    if (!ok) { next = st.tau + (F - 1.0f) / D; ok = next > st.lo && next < st.hi; }             // Newton on F
  }
  if (!ok) next = st.hi < INFINITY ? 0.5f * (st.lo + st.hi) : st.lo + 1.0f;
  const float step = next - st.tau, scale = fmaxf(1.f, fabsf(next));
  const float as = fabsf(step), ap = fabsf(st.step);
  if (as <= 3e-7f * scale) st.done = 1;
  if (order >= 2 && st.order >= 2 && as <= 0.05f * ap) {
    if (as * as * as <= 1e-7f * scale * ap * ap) st.done = 1;
    if (order == 3 && st.order == 3 && 10.f * as * as * as * as <= 1e-7f * scale * ap * ap * ap) st.done = 1;
  }
  st.step = step;
  st.order = order;
  st.tau = next;
  return st;
}

// Sum of the S slice partials (F, D) of evaluation launch k, fixed order, broadcast to the block.
__device__ __forceinline__ void sum_eval_partials(const GaussWs& ws, int k, int bh, int BH, float* bc, float& F,
                                                  float& D, float& D2) {
  const int tid = threadIdx.x;
  float f = 0.f, d = 0.f, d2 = 0.f;
  if (tid < ws.S) {
    const float* o = ws.eval_part + (((size_t)(k & 1) * BH + bh) * ws.S + tid) * 3;
    f = o[0]; d = o[1]; d2 = o[2];
  }
  if (tid < 64) { f = wave_sum(f); d = wave_sum(d); d2 = wave_sum(d2); }
  __syncthreads();
  if (tid == 0) { bc[0] = f; bc[1] = d; bc[2] = d2; }
  __syncthreads();
  F = bc[0]; D = bc[1]; D2 = bc[2];
}

template <int NB>
__global__ __launch_bounds__(kGaussEvalThreads) void gauss_eval_kernel(const float* __restrict__ mu,
                                                                       const float* __restrict__ sigma,
                                                                       const int32_t* __restrict__ seq_lens,
                                                                       GaussWs ws, int k, ZqTable zq, float margin,
                                                                       float a, int Hq, int P, int Mmax, int BH) {
  __shared__ float red[kGaussWaves][3];
  __shared__ float bc[4];
  const int bh = blockIdx.y, s = blockIdx.x, b = bh / Hq, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t lt = (1ull << lane) - 1ull;
  // Wavefront w of slice s owns the pages [wbase, wbase + pw) (cut at the end of the slice and of the sequence):
  // fixed by Mmax alone, so its first batch of (mu, sigma) is in flight before the sequence length, the
  // iteration state or the previous partials have arrived (rows have Mmax entries).
  const int wbase = s * ws.per + w * ws.pw;
  const float* mu_r = mu + (size_t)bh * Mmax;
  const float* sg_r = sigma + (size_t)bh * Mmax;
  float mv0[4], sv0[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int p = min(wbase + j * 64 + lane, Mmax - 1);
    mv0[j] = mu_r[p]; sv0[j] = sg_r[p];
  }
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const float cnt_last = (float)(n - (M - 1) * P);
  GaussState st;
  if (k == 0) {
    // start: left end from max a*mu, first point from the pooled single-Gaussian model
    HotPages hot;
    if (tid < 64) hot = load_hot_pages(ws.hot_part + (size_t)bh * ws.S * kGaussWaves * 3, ws.S * kGaussWaves);
    float mx = -INFINITY, s0 = 0.f, s1 = 0.f, s2 = 0.f;
    if (tid < ws.S) {
      const float* o = ws.init_part + ((size_t)bh * ws.S + tid) * 4;
      mx = o[0]; s0 = o[1]; s1 = o[2]; s2 = o[3];
    }
    // this lane's slice as one Gaussian of the start's mixture (lanes of wavefront 0; S <= 64)
    const float sl_n = s0, sl_m = s0 > 0.f ? s1 / s0 : 0.f;
    const float sl_sd = s0 > 0.f ? sqrtf(fmaxf(s2 / s0 - sl_m * sl_m, 0.f)) : 0.f;
    if (tid < 64) { mx = wave_max(mx); s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2); }
    if (tid == 0) { bc[0] = mx; bc[1] = s0; bc[2] = s1; bc[3] = s2; }
    __syncthreads();
    mx = bc[0]; s0 = bc[1]; s1 = bc[2]; s2 = bc[3];
    const float mean = s1 / s0;
    const float var = fmaxf(s2 / s0 - mean * mean, 0.f);
    st.lo = mx - 1.0f; st.hi = INFINITY; st.done = 0; st.step = 0.f; st.order = 0;
    // the scalar start iteration runs on one wavefront only (the others would just repeat it)
    float tau0 = 0.f;
    if (tid < 64) {
      tau0 = slice_mixture_guess<NB>(sl_n, sl_m, sl_sd, s0, mean, sqrtf(var), st.lo);
      tau0 = raise_to_hot_pages<NB>(tau0, hot);
    }
    __syncthreads();
    if (tid == 0) bc[0] = tau0;
    __syncthreads();
    st.tau = bc[0];
  } else {
    float F, D, D2;
    sum_eval_partials(ws, k - 1, bh, BH, bc, F, D, D2);
    st = advance_state(ws.state[(size_t)((k - 1) & 1) * BH + bh], F, (float)NB * D, (float)NB * D2);
  }
  if (s == 0 && tid == 0) ws.state[(size_t)(k & 1) * BH + bh] = st;
  const bool last = k == kGaussIters - 1;                 // this launch also writes the candidates
  if (st.done && !last) return;

  const int wend = min(min(wbase + ws.pw, (s + 1) * ws.per), M);
  const float thr_spec = spec_threshold(st.tau, margin);
  const float z_full = zq.z[P], z_last = zq.z[min(max(n - (M - 1) * P, 0), 64)];
  const size_t sub = ((size_t)bh * ws.S + s) * kGaussWaves + w;
  int32_t* lpage = ws.sel_page + sub * ws.pw;
  float* lkey = ws.sel_key + sub * ws.pw;
  int n_c = 0;
  float f = 0.f, d = 0.f, d2 = 0.f;
  auto batch = [&](const float (&mv)[4], const float (&sv)[4], int pb) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = pb + j * 64;
      const bool ok = p < wend;
      if (ok) {                                                        // no loads inside: divergence is harmless
        float fp, dp, dp2;
        page_mass<NB>(fmaf(a, mv[j], -st.tau), a * sv[j], p == M - 1 ? cnt_last : (float)P, fp, dp, dp2);
        f += fp; d += dp; d2 += dp2;
      }
      if (last) {                                                      // wave-uniform
        const float key = a * fmaf(sv[j], p == M - 1 ? z_last : z_full, mv[j]);
        const bool in = ok && key > thr_spec;
        const uint64_t mk = __ballot(in);
        if (in) { const int o = n_c + __popcll(mk & lt); lpage[o] = p; lkey[o] = key; }
        n_c += __popcll(mk);
      }
    }
  };
  batch(mv0, sv0, wbase + lane);                                       // the prefetched first batch
  for (int pb = wbase + 256 + lane; pb - lane < wend; pb += 256) {
    float mv[4], sv[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int p = min(pb + j * 64, Mmax - 1);                        // clamped: loads stay unconditional
      mv[j] = mu_r[p]; sv[j] = sg_r[p];
    }
    batch(mv, sv, pb);
  }
  if (last && lane == 0) ws.sel_cnt[sub] = n_c;
  f = wave_sum(f); d = wave_sum(d); d2 = wave_sum(d2);
  if (lane == 0) { red[w][0] = f; red[w][1] = d; red[w][2] = d2; }
  __syncthreads();
  if (tid == 0) {
    for (int i = 1; i < kGaussWaves; ++i) { f += red[i][0]; d += red[i][1]; d2 += red[i][2]; }
    float* o = ws.eval_part + (((size_t)(k & 1) * BH + bh) * ws.S + s) * 3;
    o[0] = f; o[1] = d; o[2] = d2;
  }
}

// Takes the last state update, keeps the candidates above the final threshold and writes them in page order.
// Rare cases are handled here by one workgroup per head: an iteration that has not converged is continued to
// convergence over all pages; if the final threshold is below the speculative one the pages are re-examined;
// nothing passed -> the single best page; more than cap pages -> the cap best estimates (lower index on
// ties), flagged.
// SINGLE: the whole selection in this one launch, for heads of a few thousand pages, where the four launches above
// are nothing but their own latencies (33 us whatever the length): the workgroup takes the pooled moments itself
// (its sixteen wavefronts own contiguous ranges of the pages and play the slices of the start's mixture, each with
// its hottest page), iterates alone over all pages -- an evaluation costs half a microsecond per 1024 pages -- and
// selects from the page estimates directly.
template <int NB, int ITEMS, bool SINGLE>
__global__ __launch_bounds__(kSelThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) void gauss_gather_kernel(
    const float* __restrict__ mu, const float* __restrict__ sigma, const int32_t* __restrict__ seq_lens,
    GaussWs ws, ZqTable zq, float margin, float a, float* __restrict__ tau_hat, int32_t* __restrict__ page_idx,
    int32_t* __restrict__ n_sel, int32_t* __restrict__ overflow, int Hq, int P, int Mmax, int cap, int BH) {
  __shared__ SelectShared sh;
  __shared__ int s_off[kGaussMaxSplits * kGaussWaves + 1];
  __shared__ int wtot[kSelWaves];
  __shared__ float red_f[kSelWaves];
  __shared__ float bc[4];
  const int bh = blockIdx.x, b = bh / Hq, tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const uint64_t lt = (1ull << lane) - 1ull;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  int32_t* out = page_idx + (size_t)bh * cap;
  if (M <= 0) { if (tid == 0) { n_sel[bh] = 0; overflow[bh] = 0; tau_hat[bh] = 0.f; } return; }
  const float cnt_last = (float)(n - (M - 1) * P);
  const float* mu_r = mu + (size_t)bh * Mmax;
  const float* sg_r = sigma + (size_t)bh * Mmax;
  GaussState st, st1;
  if (SINGLE) {
    __shared__ float w_part[kSelWaves][7];                  // per wavefront: max a*mu, count, sum, sum of squares, hottest page
    const int per_w = (M + kSelWaves - 1) / kSelWaves;      // wavefront w owns the pages [w per_w, (w+1) per_w)
    const int p_lo = w * per_w, p_hi = min(p_lo + per_w, M);
    float mx = -INFINITY, s0 = 0.f, s1 = 0.f, s2 = 0.f;
    float hk = -INFINITY, hm = 0.f, hs = 1.f, hc = 0.f;
    for (int p0 = p_lo + lane; p0 - lane < p_hi; p0 += 4 * 64) {
      float mv[4], sv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = min(p0 + j * 64, M - 1);
        mv[j] = mu_r[p]; sv[j] = sg_r[p];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = p0 + j * 64;
        if (p < p_hi) {
          const float m = a * mv[j], sd = a * sv[j];
          const float c = p == M - 1 ? cnt_last : (float)P;
          mx = fmaxf(mx, m); s0 += c; s1 = fmaf(c, m, s1); s2 = fmaf(c, fmaf(m, m, sd * sd), s2);
          const float key = fmaf(2.f, sd, m);
          if (key > hk) { hk = key; hm = m; hs = sd; hc = c; }
        }
      }
    }
    {
      const float kmax = wave_max(hk);
      const uint64_t who = __ballot(hc > 0.f && hk == kmax);
      const int src = who ? __builtin_ctzll(who) : 0;
      const float wm = __shfl(hm, src), wsd = __shfl(hs, src), wc = who ? __shfl(hc, src) : 0.f;
      mx = wave_max(mx); s0 = wave_sum(s0); s1 = wave_sum(s1); s2 = wave_sum(s2);
      if (lane == 0) {
        w_part[w][0] = mx; w_part[w][1] = s0; w_part[w][2] = s1; w_part[w][3] = s2;
        w_part[w][4] = wm; w_part[w][5] = wsd; w_part[w][6] = wc;
      }
    }
    __syncthreads();
    if (tid < 64) {
      const bool has = tid < kSelWaves;
      float pmx = has ? w_part[tid][0] : -INFINITY, c0 = has ? w_part[tid][1] : 0.f;
      float c1 = has ? w_part[tid][2] : 0.f, c2 = has ? w_part[tid][3] : 0.f;
      const float sl_n = c0, sl_m = c0 > 0.f ? c1 / c0 : 0.f;
      const float sl_sd = c0 > 0.f ? sqrtf(fmaxf(c2 / c0 - sl_m * sl_m, 0.f)) : 0.f;
      HotPages hot;
#pragma unroll
      for (int j = 0; j < 4; ++j) { hot.m[j] = 0.f; hot.s[j] = 1.f; hot.c[j] = 0.f; }
      if (has) { hot.m[0] = w_part[tid][4]; hot.s[0] = w_part[tid][5]; hot.c[0] = w_part[tid][6]; }
      pmx = wave_max(pmx); c0 = wave_sum(c0); c1 = wave_sum(c1); c2 = wave_sum(c2);
      const float mean = c1 / c0;
      const float var = fmaxf(c2 / c0 - mean * mean, 0.f);
      const float lo0 = pmx - 1.0f;
      float tau0 = slice_mixture_guess<NB>(sl_n, sl_m, sl_sd, c0, mean, sqrtf(var), lo0);
      tau0 = raise_to_hot_pages<NB>(tau0, hot);
      if (tid == 0) { bc[0] = tau0; bc[1] = lo0; }
    }
    __syncthreads();
    st.tau = bc[0]; st.lo = bc[1]; st.hi = INFINITY; st.done = 0; st.step = 0.f; st.order = 0;
    st1 = st;
  } else {
    st1 = ws.state[(size_t)((kGaussIters - 1) & 1) * BH + bh];
    float F, D, D2;
    sum_eval_partials(ws, kGaussIters - 1, bh, BH, bc, F, D, D2);
    st = advance_state(st1, F, (float)NB * D, (float)NB * D2);
  }
  int count = -1;
  for (int it = 0; it < 64 && !st.done; ++it) {            // finish the root iteration alone
    float f = 0.f, d = 0.f, d2 = 0.f;
    for (int p0 = tid; p0 < M; p0 += 4 * kSelThreads) {      // four pages per batch of loads
      float mv[4], sv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = min(p0 + j * kSelThreads, M - 1);
        mv[j] = mu_r[p]; sv[j] = sg_r[p];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = p0 + j * kSelThreads;
        if (p < M) {
          float fp, dp, dp2;
          page_mass<NB>(fmaf(a, mv[j], -st.tau), a * sv[j], p == M - 1 ? cnt_last : (float)P, fp, dp, dp2);
          f += fp; d += dp; d2 += dp2;
        }
      }
    }
    const float Fs = block_sum(f, red_f);
    const float Ds = block_sum(d, red_f);
    const float D2s = block_sum(d2, red_f);
    st = advance_state(st, Fs, (float)NB * Ds, (float)NB * D2s);
  }
  if (!SINGLE && st.tau - margin >= spec_threshold(st1.tau, margin)) {   // the candidates are complete
    const float thr = st.tau - margin;
    const int NSS = ws.S * kGaussWaves;                      // candidate lists of this head (<= 256)
    const int c = tid < NSS ? ws.sel_cnt[(size_t)bh * NSS + tid] : 0;
    int inc = c;
#pragma unroll
    for (int dd = 1; dd < 64; dd <<= 1) { const int t = __shfl_up(inc, dd); if (lane >= dd) inc += t; }
    if (lane == 63) wtot[w] = inc;
    __syncthreads();
    int base = 0, n_c = 0;
    for (int i = 0; i < kSelWaves; ++i) { const int ci = wtot[i]; if (i < w) base += ci; n_c += ci; }
    if (tid < NSS) s_off[tid] = base + inc - c;
    if (tid == 0) s_off[NSS] = n_c;
    __syncthreads();
    int n_out = 0;
    for (int e0 = 0; e0 < n_c; e0 += kSelThreads) {
      const int e = e0 + tid;
      int page = 0; bool in = false;
      if (e < n_c) {
        int lo = 0, hi = NSS;                                // invariant: s_off[lo] <= e < s_off[hi]
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_off[mid] <= e) lo = mid; else hi = mid; }
        const size_t at = ((size_t)bh * NSS + lo) * ws.pw + (e - s_off[lo]);
        page = ws.sel_page[at];
        in = ws.sel_key[at] > thr;
      }
      const uint64_t mk = __ballot(in);
      if (lane == 0) wtot[w] = __popcll(mk);
      __syncthreads();
      int off = n_out, tot = 0;
      for (int i = 0; i < kSelWaves; ++i) { const int ci = wtot[i]; if (i < w) off += ci; tot += ci; }
      const int o = off + __popcll(mk & lt);
      if (in && o < cap) out[o] = page;
      n_out += tot;
      __syncthreads();
    }
    count = n_out;
    if (count >= 1 && count <= cap) {
      if (tid == 0) { tau_hat[bh] = st.tau; n_sel[bh] = count; overflow[bh] = 0; }
      return;
    }
    if (count > cap) {
      // More pages pass than the list holds: the cap best estimates are among the candidates (every passing page
      // is one), so they are selected there -- candidate j of the concatenated lists plays the page -- instead of
      // over all pages of the head; the selected candidate numbers are then replaced by their pages.
      auto cand_at = [&](int j) {
        int lo = 0, hi = NSS;                                // invariant: s_off[lo] <= j < s_off[hi]
        while (hi - lo > 1) { const int mid = (lo + hi) >> 1; if (s_off[mid] <= j) lo = mid; else hi = mid; }
        return ((size_t)bh * NSS + lo) * ws.pw + (j - s_off[lo]);
      };
      auto ckey = [&](int j) { return float_to_key(ws.sel_key[cand_at(j)]); };
      KeySet<0, decltype(ckey)> cs(ckey, n_c);
      uint32_t vT; int k_eq;
      __syncthreads();
      radix_select_kth(cs, cap, sh, vT, k_eq);
      compact_ordered(cs, vT, k_eq, sh, out);
      __syncthreads();
      for (int e = tid; e < cap; e += kSelThreads) out[e] = ws.sel_page[cand_at(out[e])];
      if (tid == 0) { tau_hat[bh] = st.tau; n_sel[bh] = cap; overflow[bh] = 1; }
      return;
    }
  }
  if (tid == 0) tau_hat[bh] = st.tau;
  const float z_full = zq.z[P], z_last = zq.z[n - (M - 1) * P];
  auto keyfn = [=](int p) { return float_to_key(a * fmaf(sg_r[p], p == M - 1 ? z_last : z_full, mu_r[p])); };
  KeySet<ITEMS, decltype(keyfn)> ks(keyfn, M);
  if (count < 0) {                                         // the candidates were not usable: count here
    const uint32_t kthr = float_to_key(st.tau - margin);
    int c = 0;
    if constexpr (ITEMS == 0) {
      for (int i0 = 0; i0 < ks.items; i0 += 8) {
        uint32_t kb[8];
        ks.key_batch(i0, kb);
#pragma unroll
        for (int j = 0; j < 8; ++j) c += i0 + j < ks.items && kb[j] > kthr;
      }
    } else {
#pragma unroll
      for (int i = 0; i < (ITEMS ? ITEMS : ks.items); ++i) c += ks.key(i) > kthr;
    }
    count = block_sum_i(c, sh.scan_buf);
    if (count >= 1 && count <= cap) {
      compact_ordered(ks, kthr, 0, sh, out);
      if (tid == 0) { n_sel[bh] = count; overflow[bh] = 0; }
      return;
    }
  }
  const int k = count == 0 ? 1 : cap;
  uint32_t vT; int k_eq;
  radix_select_kth(ks, k, sh, vT, k_eq);
  compact_ordered(ks, vT, k_eq, sh, out);
  if (tid == 0) { n_sel[bh] = k; overflow[bh] = count > cap; }
}

static int gauss_splits(const Dims& dm) {
  const int BH = dm.B * dm.Hq;
  // about four pages per thread (one batch of loads): fewer, longer slices lose to the per-workgroup cost of
  // reading the state and reducing the partial sums (4 us on the 128K-token batch of 4), shorter ones gain nothing
  int S = (dm.Mmax + 4 * kGaussEvalThreads - 1) / (4 * kGaussEvalThreads);
  const int max_by_pages = (dm.Mmax + kGaussEvalThreads - 1) / kGaussEvalThreads;   // >= 256 pages per slice
  const int fill = (256 + BH - 1) / BH;                  // short rows: still a workgroup per compute unit
  if (S < fill) S = fill;
  if (S > max_by_pages) S = max_by_pages;
  if (S > kGaussMaxSplits) S = kGaussMaxSplits;
  if (S < 1) S = 1;
  return S;
}
static int gauss_per(const Dims& dm, int S) { return (dm.Mmax + S - 1) / S; }
static int gauss_pw(const Dims& dm, int S) { return (gauss_per(dm, S) + kGaussWaves - 1) / kGaussWaves; }

size_t select_gauss_ws_bytes(const Dims& dm) {
  const size_t BH = (size_t)dm.B * dm.Hq, S = gauss_splits(dm), pw = gauss_pw(dm, (int)S);
  size_t b = 2 * BH * sizeof(GaussState) + BH * S * 4 * sizeof(float) + 2 * BH * S * 3 * sizeof(float) +
             BH * S * kGaussWaves * 3 * sizeof(float) + BH * S * kGaussWaves * sizeof(int32_t) + BH * S * kGaussWaves * pw * (sizeof(int32_t) + sizeof(float));
  return (b + 255) & ~(size_t)255;
}

bool select_gauss_supported(const Dims& dm) { return dm.Mmax <= 4194304; }

template <int NB>
static void launch_gauss_NB(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                            const ZqTable& zq, float margin, float* tau_hat, int32_t* page_idx, int32_t* n_sel,
                            int32_t* overflow, const GaussWs& ws, hipStream_t st) {
  const int BH = dm.B * dm.Hq;
  dim3 hgrid(BH), hblock(kSelThreads);
  if (BH <= kGaussSingleRows && dm.Mmax <= kGaussSinglePages) {     // short heads: one launch does it all
    if (dm.Mmax <= 4 * kSelThreads)
      hipLaunchKernelGGL((gauss_gather_kernel<NB, 4, true>), hgrid, hblock, 0, st, mu, sigma, seq_lens, ws, zq, margin,
                         dm.a, tau_hat, page_idx, n_sel, overflow, dm.Hq, dm.P, dm.Mmax, dm.cap, BH);
    else
      hipLaunchKernelGGL((gauss_gather_kernel<NB, 16, true>), hgrid, hblock, 0, st, mu, sigma, seq_lens, ws, zq, margin,
                         dm.a, tau_hat, page_idx, n_sel, overflow, dm.Hq, dm.P, dm.Mmax, dm.cap, BH);
    return;
  }
  dim3 egrid(ws.S, BH), eblock(kGaussEvalThreads);
  hipLaunchKernelGGL(gauss_init_kernel, egrid, eblock, 0, st, mu, sigma, seq_lens, ws, dm.a, dm.Hq, dm.P, dm.Mmax);
  for (int k = 0; k < kGaussIters; ++k)
    hipLaunchKernelGGL(gauss_eval_kernel<NB>, egrid, eblock, 0, st, mu, sigma, seq_lens, ws, k, zq, margin, dm.a,
                       dm.Hq, dm.P, dm.Mmax, BH);
#define EKV_GGATHER(ITEMS)                                                                                          \
  hipLaunchKernelGGL((gauss_gather_kernel<NB, ITEMS, false>), hgrid, hblock, 0, st, mu, sigma, seq_lens, ws, zq, margin, dm.a, \
                     tau_hat, page_idx, n_sel, overflow, dm.Hq, dm.P, dm.Mmax, dm.cap, BH)
  if (dm.Mmax <= 4 * kSelThreads) EKV_GGATHER(4);
  else if (dm.Mmax <= 16 * kSelThreads) EKV_GGATHER(16);
  else EKV_GGATHER(0);
#undef EKV_GGATHER
}

void launch_select_gauss(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                         const float* zq_table, float margin, float* tau_hat, int32_t* page_idx,
                         int32_t* n_sel, int32_t* overflow, void* workspace, hipStream_t st) {
  ZqTable zq;
  for (int i = 0; i < 65; ++i) zq.z[i] = zq_table[i];
  const size_t BH = (size_t)dm.B * dm.Hq;
  GaussWs ws;
  ws.S = gauss_splits(dm);
  ws.per = gauss_per(dm, ws.S);
  ws.pw = gauss_pw(dm, ws.S);
  ws.state = (GaussState*)workspace;
  ws.init_part = (float*)(ws.state + 2 * BH);
  ws.eval_part = ws.init_part + BH * ws.S * 4;
  ws.hot_part = ws.eval_part + 2 * BH * ws.S * 3;
  ws.sel_cnt = (int32_t*)(ws.hot_part + BH * ws.S * kGaussWaves * 3);
  ws.sel_page = ws.sel_cnt + BH * ws.S * kGaussWaves;
  ws.sel_key = (float*)(ws.sel_page + BH * ws.S * kGaussWaves * ws.pw);
  switch (dm.ibeta) {
    case 1: launch_gauss_NB<1>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    case 2: launch_gauss_NB<2>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    case 3: launch_gauss_NB<3>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
    default: launch_gauss_NB<4>(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, ws, st); break;
  }
}

}  // namespace ekv
