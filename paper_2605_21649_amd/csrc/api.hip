// C ABI entry points (include/entmaxkv.h): argument validation, workspace carving, launches.
// Nothing here touches device data from the host or synchronises.
#include <cmath>
#include <cstring>
#include <mutex>
#include "ekv_internal.h"

namespace ekv {

static thread_local int32_t g_last_hip_error = 0;

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline bool ok_ptr(const void* p) { return p != nullptr && aligned16(p); }
static inline bool ok_ptr4(const void* p) { return p != nullptr && (reinterpret_cast<uintptr_t>(p) & 3u) == 0; }

static ekv_status make_dims(const ekv_config* cfg, Dims& dm) {
  if (cfg == nullptr) return EKV_ERR_INVALID_ARG;
  if (cfg->batch <= 0 || cfg->n_q_heads <= 0 || cfg->n_kv_heads <= 0 || cfg->head_dim <= 0 ||
      cfg->page_size <= 0 || cfg->max_pages_per_seq <= 0 || cfg->max_sel_pages <= 0)
    return EKV_ERR_INVALID_ARG;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return EKV_ERR_INVALID_ARG;
  if (!(cfg->alpha > 1.0f) || !std::isfinite(cfg->alpha) || !(cfg->scale > 0.0f) || !std::isfinite(cfg->scale))
    return EKV_ERR_INVALID_ARG;
  if (cfg->kv_dtype != EKV_F32 && cfg->kv_dtype != EKV_BF16) return EKV_ERR_UNSUPPORTED;
  if (cfg->head_dim != 128) return EKV_ERR_UNSUPPORTED;
  if (cfg->page_size % 4 != 0 || cfg->page_size < 4 || cfg->page_size > 64) return EKV_ERR_UNSUPPORTED;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G != 1 && G != 2 && G != 4 && G != 8) return EKV_ERR_UNSUPPORTED;
  if ((int64_t)cfg->max_pages_per_seq * cfg->page_size > (int64_t)1 << 30) return EKV_ERR_UNSUPPORTED;
  if (cfg->max_sel_pages > cfg->max_pages_per_seq) return EKV_ERR_INVALID_ARG;
  if (cfg->pool_kv_heads < 0 || (cfg->pool_kv_heads > 0 && cfg->pool_kv_heads < cfg->n_kv_heads)) return EKV_ERR_INVALID_ARG;
  dm.B = cfg->batch; dm.Hq = cfg->n_q_heads; dm.Hkv = cfg->n_kv_heads; dm.G = G; dm.P = cfg->page_size;
  dm.Mmax = cfg->max_pages_per_seq; dm.cap = cfg->max_sel_pages; dm.dtype = cfg->kv_dtype;
  dm.HkvPool = cfg->pool_kv_heads > 0 ? cfg->pool_kv_heads : cfg->n_kv_heads;
  dm.alpha = cfg->alpha; dm.scale = cfg->scale;
  dm.a = cfg->alpha - 1.0f;
  dm.beta = 1.0f / dm.a;
  const float rb = std::nearbyint(dm.beta);
  dm.ibeta = (std::fabs(dm.beta - rb) < 1e-5f * rb && rb >= 1.f && rb <= 4.f) ? (int)rb : 0;
  if (dm.ibeta) dm.beta = rb;
  return EKV_OK;
}

static ekv_status check_cache(const ekv_cache_view* c, bool need_v) {
  if (c == nullptr) return EKV_ERR_INVALID_ARG;
  if (!ok_ptr(c->k_pool) || (need_v && !ok_ptr(c->v_pool))) return EKV_ERR_INVALID_ARG;
  if (!ok_ptr4(c->block_table) || !ok_ptr4(c->seq_lens) || c->n_phys_pages <= 0) return EKV_ERR_INVALID_ARG;
  return EKV_OK;
}

// V rows are addressed by a 32-bit row index (phys*HkvPool + hkv)*P + tok inside the decode kernels.
static ekv_status check_pool_rows(const ekv_cache_view* c, const Dims& dm) {
  if ((int64_t)c->n_phys_pages * dm.HkvPool * dm.P > (int64_t)0x7fffffff) return EKV_ERR_UNSUPPORTED;
  return EKV_OK;
}

static ekv_status finish(hipStream_t) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) { g_last_hip_error = (int32_t)e; return EKV_ERR_HIP; }
  return EKV_OK;
}

// Phi^{-1}(p) in double by bisection on erfc (monotone; 200 halvings of [-40, 40]).
static double phi_inv(double log_p) {
  // solve log Phi(x) = log_p ; work with the upper tail 1 - Phi(x) = -expm1(log_p) when p is near 1
  const double upper = -std::expm1(log_p);            // 1 - p, accurate for p -> 1
  double lo = -40.0, hi = 40.0;
  for (int i = 0; i < 200; ++i) {
    const double mid = 0.5 * (lo + hi);
    const double tail = 0.5 * std::erfc(mid * M_SQRT1_2);   // 1 - Phi(mid)
    if (tail > upper) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

}  // namespace ekv

using namespace ekv;

// box (Eq. 9 on cache-dtype bounds), gauss, both, box8 (Eq. 9 on the 8-bit bounds); box or box8 may be reduced to
// the group maximum
static bool score_mode_ok(int32_t mode) {
  return (mode >= 1 && mode <= 3) || mode == (EKV_SCORE_BOX | EKV_SCORE_GROUP_MAX) || mode == EKV_SCORE_BOX8 ||
         mode == (EKV_SCORE_BOX8 | EKV_SCORE_GROUP_MAX);
}
// the optional 8-bit bounds: 16-byte units, bf16 caches only
static ekv_status check_box8(const Dims& dm, const ekv_stats_view* stats, bool required) {
  if (stats->box8 == nullptr) return required ? EKV_ERR_INVALID_ARG : EKV_OK;
  if (!aligned16(stats->box8)) return EKV_ERR_INVALID_ARG;
  return dm.dtype == EKV_BF16 ? EKV_OK : EKV_ERR_UNSUPPORTED;
}

extern "C" {

int32_t ekv_version(void) { return 102; }

int32_t ekv_last_hip_error(void) { return g_last_hip_error; }

const char* ekv_status_string(int32_t s) {
  switch (s) {
    case EKV_OK: return "EKV_OK";
    case EKV_ERR_INVALID_ARG: return "EKV_ERR_INVALID_ARG";
    case EKV_ERR_UNSUPPORTED: return "EKV_ERR_UNSUPPORTED";
    case EKV_ERR_WORKSPACE: return "EKV_ERR_WORKSPACE";
    case EKV_ERR_HIP: return "EKV_ERR_HIP";
    default: return "EKV_ERR_UNKNOWN";
  }
}

ekv_status ekv_workspace_bytes(const ekv_config* cfg, int32_t op, size_t* bytes) {
  Dims dm;
  const ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (bytes == nullptr) return EKV_ERR_INVALID_ARG;
  size_t b = 0;
  switch (op) {
    case EKV_OP_SELECT_TOPK: b = select_topk_ws_bytes(dm); break;
    case EKV_OP_SELECT_GAUSS: b = select_gauss_ws_bytes(dm); break;
    case EKV_OP_DECODE_SPARSE: b = decode_ws_carve(dm, false, nullptr, nullptr); break;
    case EKV_OP_DECODE_FULL: b = decode_ws_carve(dm, true, nullptr, nullptr); break;
    case EKV_OP_DECODE_SPARSE_SOFTMAX: b = softmax_ws_bytes(dm); break;
    case EKV_OP_SELECT_BOX_THRESHOLD:
      if (!select_box_supported(dm)) return EKV_ERR_UNSUPPORTED;
      b = select_box_ws_bytes(dm);
      break;
    default: return EKV_ERR_INVALID_ARG;
  }
  *bytes = b;
  return EKV_OK;
}

ekv_status ekv_stats_build(const ekv_config* cfg, const ekv_cache_view* cache, const ekv_stats_view* stats,
                           void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if ((s = check_cache(cache, false)) != EKV_OK) return s;
  if (stats == nullptr || !ok_ptr(stats->box) || !ok_ptr(stats->gauss)) return EKV_ERR_INVALID_ARG;
  if ((s = check_box8(dm, stats, false)) != EKV_OK) return s;
  launch_stats_build(dm, *cache, *stats, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_stats_append(const ekv_config* cfg, const ekv_cache_view* cache, const ekv_stats_view* stats,
                            const void* k_new, const void* v_new, void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if ((s = check_cache(cache, v_new != nullptr)) != EKV_OK) return s;
  if (stats == nullptr || !ok_ptr(stats->box) || !ok_ptr(stats->gauss)) return EKV_ERR_INVALID_ARG;
  if (!ok_ptr(k_new) || (v_new != nullptr && !aligned16(v_new))) return EKV_ERR_INVALID_ARG;
  if ((s = check_box8(dm, stats, false)) != EKV_OK) return s;
  launch_stats_append(dm, *cache, *stats, k_new, v_new, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_score_pages(const ekv_config* cfg, const void* q, const ekv_stats_view* stats,
                           const int32_t* seq_lens, int32_t mode, float* box, float* mu, float* sigma,
                           void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (!score_mode_ok(mode) || !ok_ptr(q) || stats == nullptr || !ok_ptr4(seq_lens)) return EKV_ERR_INVALID_ARG;
  if ((mode & EKV_SCORE_BOX) && (!ok_ptr(stats->box) || !ok_ptr4(box))) return EKV_ERR_INVALID_ARG;
  if (mode & EKV_SCORE_BOX8) {
    if (!ok_ptr4(box)) return EKV_ERR_INVALID_ARG;
    if ((s = check_box8(dm, stats, true)) != EKV_OK) return s;
  }
  if ((mode & EKV_SCORE_GAUSS) && (!ok_ptr(stats->gauss) || !ok_ptr4(mu) || !ok_ptr4(sigma)))
    return EKV_ERR_INVALID_ARG;
  launch_score_pages(dm, q, *stats, seq_lens, mode, box, mu, sigma, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_append_score_pages(const ekv_config* cfg, const ekv_cache_view* cache, const ekv_stats_view* stats,
                                  const void* k_new, const void* v_new, const void* q, int32_t mode, float* box,
                                  float* mu, float* sigma, void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if ((s = check_cache(cache, false)) != EKV_OK) return s;
  if (v_new != nullptr && !ok_ptr(cache->v_pool)) return EKV_ERR_INVALID_ARG;
  if (!score_mode_ok(mode) || !ok_ptr(q) || !ok_ptr(k_new) || (v_new != nullptr && !ok_ptr(v_new)))
    return EKV_ERR_INVALID_ARG;
  if (stats == nullptr || !ok_ptr(stats->box) || !ok_ptr(stats->gauss)) return EKV_ERR_INVALID_ARG;
  if ((s = check_box8(dm, stats, (mode & EKV_SCORE_BOX8) != 0)) != EKV_OK) return s;
  if ((mode & (EKV_SCORE_BOX | EKV_SCORE_BOX8)) && !ok_ptr4(box)) return EKV_ERR_INVALID_ARG;
  if ((mode & EKV_SCORE_GAUSS) && (!ok_ptr4(mu) || !ok_ptr4(sigma))) return EKV_ERR_INVALID_ARG;
  launch_score_pages(dm, q, *stats, cache->seq_lens, mode, box, mu, sigma, (hipStream_t)stream, cache, k_new, v_new);
  return finish((hipStream_t)stream);
}

ekv_status ekv_select_topk(const ekv_config* cfg, const float* box, const int32_t* seq_lens, int32_t k_pages,
                           int32_t* page_idx, int32_t* n_sel, void* workspace, size_t workspace_bytes,
                           void* stream) {
  Dims dm;
  const ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (!ok_ptr4(box) || !ok_ptr4(seq_lens) || !ok_ptr4(page_idx) || !ok_ptr4(n_sel)) return EKV_ERR_INVALID_ARG;
  if (k_pages < 1 || k_pages > dm.cap) return EKV_ERR_INVALID_ARG;
  if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < select_topk_ws_bytes(dm))
    return EKV_ERR_WORKSPACE;
  launch_select_topk(dm, box, seq_lens, k_pages, page_idx, n_sel, workspace, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_select_gauss(const ekv_config* cfg, const float* mu, const float* sigma, const int32_t* seq_lens,
                            float q_page, float margin, float* tau_hat, int32_t* page_idx, int32_t* n_sel,
                            int32_t* overflow, void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  const ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (dm.ibeta == 0 || !select_gauss_supported(dm)) return EKV_ERR_UNSUPPORTED;
  if (!ok_ptr4(mu) || !ok_ptr4(sigma) || !ok_ptr4(seq_lens) || !ok_ptr4(tau_hat) || !ok_ptr4(page_idx) ||
      !ok_ptr4(n_sel) || !ok_ptr4(overflow))
    return EKV_ERR_INVALID_ARG;
  if (!(q_page > 0.f && q_page < 1.f) || !(margin >= 0.f) || !std::isfinite(margin)) return EKV_ERR_INVALID_ARG;
  if (workspace == nullptr || workspace_bytes < select_gauss_ws_bytes(dm)) return EKV_ERR_WORKSPACE;
  // PhiInv(q_page^(1/c)), Eq. 11, for every possible page fill c; cached per thread for the last q_page
  static thread_local float zq[65];
  static thread_local float zq_for = -1.f;
  if (zq_for != q_page) {
    zq[0] = 0.f;
    const double lq = std::log((double)q_page);
    for (int c = 1; c <= 64; ++c) zq[c] = (float)phi_inv(lq / (double)c);
    zq_for = q_page;
  }
  launch_select_gauss(dm, mu, sigma, seq_lens, zq, margin, tau_hat, page_idx, n_sel, overflow, workspace,
                      (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_select_box_threshold(const ekv_config* cfg, const float* box, const int32_t* seq_lens,
                                    const float* tau_lo, const int32_t* page_idx_in, const int32_t* n_sel_in,
                                    int32_t* page_idx_out, int32_t* n_sel_out, int32_t* n_added, int32_t* overflow,
                                    void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  const ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (!select_box_supported(dm)) return EKV_ERR_UNSUPPORTED;
  if (!ok_ptr4(box) || !ok_ptr4(seq_lens) || !ok_ptr4(tau_lo) || !ok_ptr4(page_idx_out) || !ok_ptr4(n_sel_out) ||
      !ok_ptr4(n_added) || !ok_ptr4(overflow))
    return EKV_ERR_INVALID_ARG;
  if ((page_idx_in == nullptr) != (n_sel_in == nullptr)) return EKV_ERR_INVALID_ARG;
  if (page_idx_in != nullptr && (!ok_ptr4(page_idx_in) || !ok_ptr4(n_sel_in))) return EKV_ERR_INVALID_ARG;
  if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < select_box_ws_bytes(dm))
    return EKV_ERR_WORKSPACE;
  launch_select_box_threshold(dm, box, seq_lens, tau_lo, page_idx_in, n_sel_in, page_idx_out, n_sel_out, n_added,
                              overflow, workspace, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

static ekv_status decode_common(const ekv_config* cfg, bool dense, bool grouped, const void* q, const ekv_cache_view* cache,
                                const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                                int32_t* supp, const ekv_decode_extras* extras, void* workspace,
                                size_t workspace_bytes, void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if ((s = check_cache(cache, true)) != EKV_OK) return s;
  if ((s = check_pool_rows(cache, dm)) != EKV_OK) return s;
  if (!ok_ptr(q) || !ok_ptr4(out) || !ok_ptr4(tau) || !ok_ptr4(supp)) return EKV_ERR_INVALID_ARG;
  if (!dense && (!ok_ptr4(page_idx) || !ok_ptr4(n_sel))) return EKV_ERR_INVALID_ARG;
  ekv_decode_extras ex;
  std::memset(&ex, 0, sizeof(ex));
  if (extras != nullptr) {
    ex = *extras;
    if (ex.support_tokens != nullptr && ex.support_cap <= 0) return EKV_ERR_INVALID_ARG;
    if (!dense) ex.lse = nullptr;
  }
  DecodeWorkspace ws;
  const size_t need = decode_ws_carve(dm, dense, nullptr, nullptr);
  if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < need) return EKV_ERR_WORKSPACE;
  decode_ws_carve(dm, dense, workspace, &ws);
  launch_decode(dm, dense, grouped, q, *cache, page_idx, n_sel, out, tau, supp, ex, ws, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_decode_sparse(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                             const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau, int32_t* supp,
                             const ekv_decode_extras* extras, void* workspace, size_t workspace_bytes,
                             void* stream) {
  return decode_common(cfg, false, false, q, cache, page_idx, n_sel, out, tau, supp, extras, workspace,
                       workspace_bytes, stream);
}

// ---- entry point that allocates nothing: decode scratch in a static device array -------------------------------
// A __device__ array is part of the code object: every GPU the library is loaded on holds its own copy, at its own
// address, until the process ends.  In host code the array's name only stands for the symbol; its device address is
// looked up once per device and only that address is used afterwards.
namespace ekv {
constexpr size_t kStaticScratchBytes = (size_t)EKV_STATIC_SCRATCH_BYTES;
constexpr int kStaticScratchDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kStaticScratchDevices] = {nullptr};
static std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch` (looked up on the first call on a device, with that device current).
static ekv_status static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) { g_last_hip_error = (int32_t)e; return EKV_ERR_HIP; }
  if (dev < 0 || dev >= kStaticScratchDevices) return EKV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || ptr == nullptr) { g_last_hip_error = (int32_t)e; return EKV_ERR_HIP; }
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return EKV_OK;
}
}  // namespace ekv

ekv_status ekv_decode_sparse_static(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                                    const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                                    int32_t* supp, const ekv_decode_extras* extras, void* stream) {
  Dims dm;
  const ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if (decode_ws_carve(dm, false, nullptr, nullptr) > kStaticScratchBytes) return EKV_ERR_WORKSPACE;
  void* ws = nullptr;
  const ekv_status ss = static_scratch(&ws);
  if (ss != EKV_OK) return ss;
  return decode_common(cfg, false, false, q, cache, page_idx, n_sel, out, tau, supp, extras, ws, kStaticScratchBytes,
                       stream);
}

ekv_status ekv_decode_full(const ekv_config* cfg, const void* q, const ekv_cache_view* cache, float* out,
                           float* tau, int32_t* supp, const ekv_decode_extras* extras, void* workspace,
                           size_t workspace_bytes, void* stream) {
  return decode_common(cfg, true, false, q, cache, nullptr, nullptr, out, tau, supp, extras, workspace,
                       workspace_bytes, stream);
}

ekv_status ekv_decode_sparse_group(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                                   const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                                   int32_t* supp, const ekv_decode_extras* extras, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return decode_common(cfg, false, true, q, cache, page_idx, n_sel, out, tau, supp, extras, workspace,
                       workspace_bytes, stream);
}

ekv_status ekv_decode_sparse_softmax(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                                     const int32_t* page_idx, const int32_t* n_sel, float* out, float* lse_sel,
                                     void* workspace, size_t workspace_bytes, void* stream) {
  Dims dm;
  ekv_status s = make_dims(cfg, dm);
  if (s != EKV_OK) return s;
  if ((s = check_cache(cache, true)) != EKV_OK) return s;
  if (!ok_ptr(q) || !ok_ptr4(page_idx) || !ok_ptr4(n_sel) || !ok_ptr4(out) || !ok_ptr4(lse_sel))
    return EKV_ERR_INVALID_ARG;
  if (workspace == nullptr || !aligned16(workspace) || workspace_bytes < softmax_ws_bytes(dm))
    return EKV_ERR_WORKSPACE;
  launch_decode_sparse_softmax(dm, q, *cache, page_idx, n_sel, out, lse_sel, workspace, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_probe_read(const void* base, const int32_t* page_ids, const int32_t* lookup, int32_t n_pages,
                          int32_t page_bytes, float* out, void* sink, void* stream) {
  if (!ok_ptr(base) || !ok_ptr4(page_ids) || !ok_ptr4(sink) || n_pages <= 0) return EKV_ERR_INVALID_ARG;
  if ((lookup != nullptr && !ok_ptr4(lookup)) || (out != nullptr && !ok_ptr4(out))) return EKV_ERR_INVALID_ARG;
  if (page_bytes != 4096 && page_bytes != 8192) return EKV_ERR_UNSUPPORTED;
  launch_probe_read(base, page_ids, lookup, n_pages, page_bytes, out, (uint32_t*)sink, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

ekv_status ekv_probe_handoff(float* data, uint32_t* counter, float* out, int32_t n_workgroups, int32_t mode,
                             void* stream) {
  if (!ok_ptr4(data) || !ok_ptr4(counter) || !ok_ptr4(out)) return EKV_ERR_INVALID_ARG;
  if (n_workgroups < 2 || n_workgroups > 65536 || mode < 0 || mode > 2) return EKV_ERR_INVALID_ARG;
  launch_probe_handoff(data, counter, out, n_workgroups, mode, (hipStream_t)stream);
  return finish((hipStream_t)stream);
}

}  // extern "C"
