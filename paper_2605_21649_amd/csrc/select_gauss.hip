// Gaussian-aware entmax selector (paper Sec. 4.3 Eq. 10-12, App. D).
//
// Per (sequence, query head): solve  F(tau) = sum_p cnt_p * E[(a S_p - tau)_+^beta] = 1  for tau_hat,
// S_p ~ N(mu_p, sigma_p^2), with the truncated Gaussian moments in closed form (integer beta), then
// keep the pages whose estimated maximum a*(mu_p + sigma_p*z_cnt) exceeds tau_hat - margin and write
// them in ascending order.  One 1024-thread workgroup per (b,h); mu/sigma are re-read from L2 in
// every iteration.
//
// Root finding: F is positive, decreasing and convex.  The iteration is Newton on log F (which removes
// the slow phase of plain Newton while F >> 1) kept inside a bracket [lo, hi] with F(lo) >= 1 > F(hi);
// a step that leaves the bracket is replaced by bisection.  The left end a*mu_max - 1 is valid because
// cnt*E[(Y)_+^beta] >= cnt*(E Y)_+^beta >= 1 there (Jensen).
#include "ekv_select.h"
#include "ekv_internal.h"

namespace ekv {

constexpr float kInvSqrt2 = 0.70710678118654752f;
constexpr float kInvSqrt2Pi = 0.39894228040143268f;

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
    const float phi = __expf(-0.5f * t * t) * kInvSqrt2Pi;
    float h[5];
    h[0] = Phi;
    h[1] = fmaf(t, Phi, phi);
#pragma unroll
    for (int n = 2; n <= NB; ++n) h[n] = fmaf(t, h[n - 1], (float)(n - 1) * h[n - 2]);
    h_nb = h[NB]; h_nbm1 = h[NB - 1];
  } else {
    constexpr int N = 26;
    float hn1 = 0.f, hn = 1.f;            // h_{n+1}, h_n at n = N
    float cap_nb = 0.f, cap_nbm1 = 0.f;
#pragma unroll
    for (int n = N + 1; n >= 2; --n) {    // computes h_{n-2} from (h_n = hn1 slot, h_{n-1} = hn slot)
      const float hm = (hn1 - t * hn) * (1.0f / (float)(n - 1));
      hn1 = hn; hn = hm;                  // now hn = h_{n-2}, hn1 = h_{n-1}
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

struct ZqTable { float z[65]; };   // z[c] = PhiInv(q_page^(1/c)), c = 1..64

template <int NB>
__global__ __launch_bounds__(kSelThreads) void select_gauss_kernel(
    const float* __restrict__ mu, const float* __restrict__ sigma, const int32_t* __restrict__ seq_lens,
    ZqTable zq, float margin, float a, float* __restrict__ tau_hat, int32_t* __restrict__ page_idx,
    int32_t* __restrict__ n_sel, int32_t* __restrict__ overflow, int Hq, int P, int Mmax, int cap) {
  __shared__ SelectShared sh;
  __shared__ float red_f[kSelWaves];
  const int bh = blockIdx.x, b = bh / Hq, tid = threadIdx.x;
  const int n = seq_lens[b];
  const int M = (n + P - 1) / P;
  const float cnt_last = (float)(n - (M - 1) * P);
  const float* mu_r = mu + (size_t)bh * Mmax;
  const float* sg_r = sigma + (size_t)bh * Mmax;

  float mmax = -INFINITY;
  for (int p = tid; p < M; p += kSelThreads) mmax = fmaxf(mmax, mu_r[p]);
  mmax = block_max(mmax, red_f);

  float lo = a * mmax - 1.0f, hi = INFINITY;
  float tau = lo;
  for (int it = 0; it < 64; ++it) {
    float f = 0.f, d = 0.f;
    for (int p = tid; p < M; p += kSelThreads) {
      float fp, dp;
      page_mass<NB>(fmaf(a, mu_r[p], -tau), a * sg_r[p], p == M - 1 ? cnt_last : (float)P, fp, dp);
      f += fp; d += dp;
    }
    const float F = block_sum(f, red_f);
    const float D = (float)NB * block_sum(d, red_f);         // -dF/dtau
    if (F >= 1.0f) lo = tau; else hi = tau;
    float next;
    if (F > 0.f && D > 0.f) next = tau + F * __logf(F) / D;  // Newton on log F
    else next = 0.5f * (lo + tau);                           // far right of the root: come back
    if (hi < INFINITY && !(next > lo && next < hi)) next = 0.5f * (lo + hi);
    const float step = fabsf(next - tau);
    tau = next;
    if (step <= 6e-8f * fmaxf(1.f, fabsf(tau))) break;
  }
  if (tid == 0) tau_hat[bh] = tau;

  // selection: keep p iff a*(mu_p + sigma_p z_cnt) > tau - margin
  const float thr = tau - margin;
  const float z_full = zq.z[P], z_last = zq.z[(int)cnt_last];
  auto gfn = [=](int p) { return a * fmaf(sg_r[p], p == M - 1 ? z_last : z_full, mu_r[p]); };
  auto keyfn = [=](int p) { return float_to_key(gfn(p)); };
  int c = 0;
  for (int p = tid; p < M; p += kSelThreads) c += gfn(p) > thr;
  const int count = block_sum_i(c, sh.scan_buf);
  int32_t* out = page_idx + (size_t)bh * cap;
  int n_out, ovf = 0;
  if (count >= 1 && count <= cap) {
    compact_ordered(keyfn, M, 0u, float_to_key(thr), 0, sh, out);
    n_out = count;
  } else {
    // nothing passed: the single best page; too many: the cap best pages (lower index on ties)
    const int k = count == 0 ? 1 : cap;
    ovf = count > cap;
    uint32_t kmin, vT; int k_eq;
    radix_select_kth(keyfn, M, k, sh, kmin, vT, k_eq);
    compact_ordered(keyfn, M, kmin, vT, k_eq, sh, out);
    n_out = k;
  }
  if (tid == 0) { n_sel[bh] = n_out; overflow[bh] = ovf; }
}

size_t select_gauss_ws_bytes(const Dims&) { return 256; }

void launch_select_gauss(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                         const float* zq_table, float margin, float* tau_hat, int32_t* page_idx,
                         int32_t* n_sel, int32_t* overflow, void*, hipStream_t st) {
  ZqTable zq;
  for (int i = 0; i < 65; ++i) zq.z[i] = zq_table[i];
  dim3 grid(dm.B * dm.Hq), block(kSelThreads);
#define EKV_LAUNCH_GAUSS(NB)                                                                              \
  hipLaunchKernelGGL(select_gauss_kernel<NB>, grid, block, 0, st, mu, sigma, seq_lens, zq, margin, dm.a,  \
                     tau_hat, page_idx, n_sel, overflow, dm.Hq, dm.P, dm.Mmax, dm.cap)
  switch (dm.ibeta) {
    case 1: EKV_LAUNCH_GAUSS(1); break;
    case 2: EKV_LAUNCH_GAUSS(2); break;
    case 3: EKV_LAUNCH_GAUSS(3); break;
    default: EKV_LAUNCH_GAUSS(4); break;
  }
#undef EKV_LAUNCH_GAUSS
}

}  // namespace ekv
