// Host-side launcher declarations (internal to the library).  Arguments are validated in api.hip
// before any launcher is called; launchers only enqueue kernels on the given stream.
#pragma once
#include <hip/hip_runtime.h>
#include "../../include/entmaxkv.h"

namespace ekv {

struct Dims {
  int B, Hq, Hkv, G, P, Mmax, cap;
  int HkvPool;        // KV heads per physical page of the pools (>= Hkv; the stride when a config covers a subset)
  int dtype;          // ekv_dtype
  float alpha, scale;
  float a;            // alpha - 1
  float beta;         // 1 / a
  int ibeta;          // beta if it is 1,2,3,4 (within 1e-6), else 0
};

// decode scratch layout (shared by api.hip and decode.hip)
// page slots per entry of pmax (granularity of chunk skipping): 64 tokens when P divides 64
__host__ __device__ inline int pmax_pages(int P) { return P >= 64 ? 1 : 64 / P; }

// Long rows are pre-filtered by multi-workgroup passes before the single-workgroup solve.
constexpr int kFilterSliceChunks = 512;   // pmax entries (groups of <= 64 tokens) per workgroup of the filter
constexpr int kPreGroups = 4096;          // rows of at most this many groups are solved without the filter passes
constexpr int kFilterMaxSlices = 1024;    // ... unless they would need more slices than this
constexpr int kFilterSliceCap = 4096;     // candidates kept per slice (the solve holds this many in LDS)

struct DecodeWorkspace {
  float* z;        // [B*Hq][zstride] candidate scores z_j (or -inf where masked)
  float* pmax;     // [B*Hq][n_chunks_max] maxima of z per pmax_pages(P) page slots
  int32_t* unit_pre;  // [B*Hq + 1] item prefix of pass 1 (used when the units do not fit in LDS)
  float* spill_u;      // [B*Hq][spill_cap] overflow of the solve's candidate list (z - zmax), null when rows are short
  int32_t* spill_pos;  // [B*Hq][spill_cap] positions of those candidates
  int spill_cap;
  size_t zstride;  // floats per (b,h) row of z
  int n_chunks_max;
  // filter passes; all null / 0 when the rows are short
  int n_slices_max;
  int32_t* fcount;     // [B*Hq][n_slices_max] candidates above the certified bound, per slice
  float* frow;         // [B*Hq][2]: zmax, certified lower bound of tau
  float* flist_u;      // [B*Hq][n_slices_max][kFilterSliceCap] z - zmax of those candidates, in order
  int32_t* flist_pos;  // ... and their positions
};

// Carves the decode scratch out of `base` (may be null: size query only); returns the bytes needed.
size_t decode_ws_carve(const Dims& dm, bool dense, void* base, DecodeWorkspace* ws);

void launch_stats_build(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s, hipStream_t st);
void launch_stats_append(const Dims& dm, const ekv_cache_view& c, const ekv_stats_view& s,
                         const void* k_new, const void* v_new, hipStream_t st);
// append_to != nullptr: fused append of (k_new, v_new) at slot seq_lens[b] before scoring with seq_lens[b] + 1
void launch_score_pages(const Dims& dm, const void* q, const ekv_stats_view& s, const int32_t* seq_lens,
                        int mode, float* box, float* mu, float* sigma, hipStream_t st,
                        const ekv_cache_view* append_to = nullptr, const void* k_new = nullptr,
                        const void* v_new = nullptr);
void launch_select_topk(const Dims& dm, const float* box, const int32_t* seq_lens, int k_pages,
                        int32_t* page_idx, int32_t* n_sel, void* ws, hipStream_t st);
void launch_select_gauss(const Dims& dm, const float* mu, const float* sigma, const int32_t* seq_lens,
                         const float* zq_table, float margin, float* tau_hat, int32_t* page_idx,
                         int32_t* n_sel, int32_t* overflow, void* ws, hipStream_t st);
// grouped: page_idx/n_sel have one row per (b, KV head), shared by the G query heads of the group
void launch_decode(const Dims& dm, bool dense, bool grouped, const void* q, const ekv_cache_view& c,
                   const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau, int32_t* supp,
                   const ekv_decode_extras& ex, const DecodeWorkspace& ws, hipStream_t st);
void launch_decode_sparse_softmax(const Dims& dm, const void* q, const ekv_cache_view& c,
                                  const int32_t* page_idx, const int32_t* n_sel, float* out,
                                  float* lse_sel, void* ws, hipStream_t st);

void launch_select_box_threshold(const Dims& dm, const float* box, const int32_t* seq_lens, const float* tau_lo,
                                 const int32_t* page_idx_in, const int32_t* n_sel_in, int32_t* page_idx_out,
                                 int32_t* n_sel_out, int32_t* n_added, int32_t* overflow, void* workspace,
                                 hipStream_t st);

void launch_probe_read(const void* base, const int32_t* page_ids, const int32_t* lookup, int n_pages, int page_bytes,
                       float* out, uint32_t* sink, hipStream_t st);

void launch_probe_handoff(float* data, uint32_t* counter, float* out, int n_workgroups, int mode, hipStream_t st);

size_t select_topk_ws_bytes(const Dims& dm);
size_t select_box_ws_bytes(const Dims& dm);
bool select_box_supported(const Dims& dm);
size_t select_gauss_ws_bytes(const Dims& dm);
bool select_gauss_supported(const Dims& dm);
size_t softmax_ws_bytes(const Dims& dm);

}  // namespace ekv
