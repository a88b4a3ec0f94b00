/* entmaxkv.h -- C ABI of the MI355X (gfx950) decode hot path of EntmaxKV:
 * support-aware sparse alpha-entmax attention over a paged KV cache.
 *
 * One decode step (paper Sec. 4.1, Sec. 4.4) is, per sequence b and query head h:
 *   stats (build once / append per token) -> score pages -> select pages -> sparse entmax decode,
 * with a dense full-cache entmax decode alongside as the baseline.
 *
 * Conventions (all entry points):
 *  - plain C, no exceptions; every call returns an ekv_status.
 *  - every pointer named in a *_view or marked "device" is a DEVICE pointer owned by the caller,
 *    16-byte aligned; the library allocates no device memory.  Scratch comes from the caller's
 *    workspace (size from ekv_workspace_bytes).  Config structs are HOST pointers.
 *  - calls enqueue kernels on `stream` (a hipStream_t passed as void*; NULL = default stream) and
 *    return without synchronising; no device data is read on the host.
 *  - variable-length results are (indices, count) pairs on the device with fixed capacity.
 *  - the same inputs give bit-identical outputs from run to run (fixed reduction orders, no
 *    floating-point atomics).
 *  - outputs must not alias inputs, unless an entry point says otherwise.
 *
 * Shapes use: B batch, Hq query heads, Hkv KV heads, G=Hq/Hkv, d head_dim (=128), P page_size,
 * Mmax = max_pages_per_seq, cap = max_sel_pages, n_b = seq_lens[b], M_b = ceil(n_b/P),
 * a = alpha-1, beta = 1/a.  Query head h reads KV head h / G.
 */
#ifndef ENTMAXKV_H
#define ENTMAXKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EKV_OK = 0,
  EKV_ERR_INVALID_ARG = 1, /* null/misaligned pointer, non-positive size, inconsistent config      */
  EKV_ERR_UNSUPPORTED = 2, /* head_dim / page_size / dtype / alpha this build has no kernel for,   */
                           /* or a size beyond a kernel's range (stated with each entry point)      */
  EKV_ERR_WORKSPACE = 3,   /* workspace pointer NULL or smaller than ekv_workspace_bytes reports   */
  EKV_ERR_HIP = 4          /* a HIP runtime call failed; ekv_last_hip_error() returns its code     */
} ekv_status;

typedef enum { EKV_F32 = 0, EKV_BF16 = 1 } ekv_dtype;

/* Which page scores ekv_score_pages writes. */
typedef enum {
  EKV_SCORE_BOX = 1,
  EKV_SCORE_GAUSS = 2,
  EKV_SCORE_BOTH = 3,
  EKV_SCORE_GROUP_MAX = 4, /* with EKV_SCORE_BOX or EKV_SCORE_BOX8 only: one score per KV head, the maximum over
                              its query heads */
  EKV_SCORE_BOX8 = 8       /* the box score computed from the 8-bit bounds stats->box8 (alone or with GROUP_MAX) */
} ekv_score_mode;

/* Operations a workspace can be sized for. */
typedef enum {
  EKV_OP_SELECT_TOPK = 0,
  EKV_OP_SELECT_GAUSS = 1,
  EKV_OP_DECODE_SPARSE = 2,
  EKV_OP_DECODE_FULL = 3,
  EKV_OP_DECODE_SPARSE_SOFTMAX = 4,
  EKV_OP_SELECT_BOX_THRESHOLD = 5
} ekv_op;

/* Problem description (host struct).  head_dim must be 128; page_size a multiple of 4 in [4,64];
 * n_q_heads a multiple of n_kv_heads with G in {1,2,4,8}; alpha > 1 (beta = 1/(alpha-1) need not
 * be an integer for the decode calls; ekv_select_gauss needs beta in {1,2,3,4}, paper App. D). */
typedef struct {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t page_size;
  int32_t kv_dtype;          /* ekv_dtype of K/V pools, q and the page statistics                  */
  float alpha;               /* entmax alpha (paper Eq. 2)                                         */
  float scale;               /* score multiplier; the paper's 1/sqrt(d) (Eq. 1)                    */
  int32_t max_pages_per_seq; /* Mmax: row length of block_table and of the per-page score arrays   */
  int32_t max_sel_pages;     /* cap: row length of page_idx.  It sizes workspaces only: the time   */
                             /* of the decode calls follows the lists' device-side lengths         */
  int32_t pool_kv_heads;     /* KV heads per physical page of the pools; 0 means n_kv_heads.  A     */
                             /* config may cover only heads [h0, h0 + n_kv_heads) of a cache with   */
                             /* more heads (to run independent head groups on separate streams):    */
                             /* set this to the cache's head count, pass k_pool / v_pool advanced   */
                             /* by h0*P*d elements, and every [B][H..] array restricted to those     */
                             /* heads (contiguous slices when batch == 1)                           */
} ekv_config;

/* Paged KV cache (paper Sec. 4.2: block layout of PagedAttention).  Physical page `phys` of KV head h
 * is the contiguous block pool[((phys*pool_kv_heads + h)*P + t)*d + i], t < P, i < d, element type kv_dtype.
 * block_table[b*Mmax + p] = physical page of logical page p of sequence b (0 <= phys < n_phys_pages;
 * entries with p >= M_b may hold anything: what is read from them is clamped into range and masked).
 * seq_lens[b] = n_b >= 0.  A sequence with n_b = 0 (an idle slot of a serving batch) is legal in every call:
 * its score rows are all -inf (sigma 0), the selectors return no page (tau_hat 0), the decodes write a zero
 * output, tau = +inf, an empty support, and a log-sum-exp of -inf; an append makes it a sequence of one token. */
typedef struct {
  void* k_pool;
  void* v_pool;
  const int32_t* block_table;
  const int32_t* seq_lens;
  int32_t n_phys_pages;
} ekv_cache_view;

/* Page statistics (paper Sec. 4.2), stored per SEQUENCE in logical page order so that scoring is a
 * pure stream:  box  [B][Hkv][Mmax][2][d]  = (k_min, k_max)   element-wise over the page's tokens,
 *               gauss[B][Hkv][Mmax][2][d]  = (k_avg, k_var)   population mean and variance k_std^2,
 * both in kv_dtype.  (The variance rather than k_std is stored because sigma_p^2 of Sec. 4.3 is linear
 * in it, which lets the scoring kernel run as one bf16 matrix contraction; k_std = sqrt(k_var).)
 * Rows of pages p >= M_b are not defined.  Either pointer may be NULL in calls that do not need it
 * (scoring with a mode that does not read it).
 * box8 (optional, may be NULL everywhere): the same bounds in 8 bits per value, half the bytes to stream
 * when scoring -- an extension; the paper keeps its metadata in the cache dtype.  uint8 [B][Hkv][Mmax][16][2][8]:
 * unit u of a page holds k_min of channels 8u..8u+7, then k_max of the same channels, as OCP E4M3 codes
 * (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; 0x7f/0xff = NaN; largest finite value 448), with
 * k_min rounded DOWN and k_max rounded UP to the format, so that Eq. 9 computed from them is still an upper
 * bound of every token score of the page (only looser).  A bound the format cannot hold (k_max > 448,
 * k_min < -448, NaN) is stored as NaN and gives the page the score +inf: it is always selected.
 * kv_dtype must be EKV_BF16.  When box8 is not NULL, ekv_stats_build, ekv_stats_append and
 * ekv_append_score_pages keep it up to date together with box and gauss. */
typedef struct {
  void* box;
  void* gauss;
  void* box8;
} ekv_stats_view;

/* a1 -- bulk statistics build (Sec. 4.2).  For every sequence b, KV head and logical page p < M_b,
 * computes k_min, k_max, k_avg and k_var = max(m2 - k_avg^2, 0) (= k_std^2) over the page's cnt tokens
 * (cnt = P, or n_b - pP for the last page) and writes both stats arrays (both must be non-NULL). */
ekv_status ekv_stats_build(const ekv_config* cfg, const ekv_cache_view* cache,
                           const ekv_stats_view* stats, void* stream);

/* a2 -- append one token per sequence and bring its page's statistics up to date (Sec. 4.2).
 * k_new [B][Hkv][d] (device, kv_dtype) is written to slot n_b of the cache (logical page n_b/P,
 * token n_b%P; that page must already be mapped in block_table and n_b < Mmax*P); v_new likewise
 * when not NULL.  The statistics of that page are recomputed over its n_b%P + 1 tokens with the
 * same arithmetic as ekv_stats_build, so append-then-query equals rebuild-then-query bit for bit.
 * seq_lens is NOT modified: the caller adds 1 to every entry after this call. */
ekv_status ekv_stats_append(const ekv_config* cfg, const ekv_cache_view* cache,
                            const ekv_stats_view* stats, const void* k_new, const void* v_new,
                            void* stream);

/* a3/a4 -- query-aware page scoring (Sec. 4.2 Eq. 9; Sec. 4.3 page moments).
 * q [B][Hq][d] device, kv_dtype.  Outputs, each f32 [B][Hq][Mmax] (device) or NULL if not requested:
 *   box[b,h,p]   = scale * sum_i max(q_i kmin_i, q_i kmax_i)          (mode & EKV_SCORE_BOX)
 *   mu[b,h,p]    = scale * q . k_avg                                   (mode & EKV_SCORE_GAUSS)
 *   sigma[b,h,p] = scale * sqrt(sum_i q_i^2 k_var,i)                   (mode & EKV_SCORE_GAUSS)
 * Entries p >= M_b are written as -inf (box, mu) and 0 (sigma).
 * mode == EKV_SCORE_BOX8 computes box from stats->box8 instead (bf16 only; not combined with BOX or GAUSS
 * in one call); pages with a NaN bound score +inf.
 * mode == EKV_SCORE_BOX | EKV_SCORE_GROUP_MAX writes instead box f32 [B][Hkv][Mmax], the maximum of the G
 * query heads' box scores of each KV head: the score of a page list shared by the group (the paper
 * selects per attention head and does not treat grouped-query attention; the maximum keeps Eq. 9 an
 * upper bound for every head of the group).  Select on it with a config whose n_q_heads equals
 * n_kv_heads (ekv_select_topk and ekv_select_box_threshold have batch x n_q_heads rows), then decode with
 * ekv_decode_sparse_group. */
ekv_status ekv_score_pages(const ekv_config* cfg, const void* q, const ekv_stats_view* stats,
                           const int32_t* seq_lens, int32_t mode, float* box, float* mu,
                           float* sigma, void* stream);

/* a2 + a3/a4 in one call: ekv_stats_append followed by ekv_score_pages over the lengths n_b + 1, bit for bit.
 * For pages of up to 32 tokens it is one launch, without the separate small launch of the append on the
 * critical path of a decode step: a workgroup of the scoring kernel appends the token first (cache slot
 * written, that page's statistics recomputed) and scores the tile of that page, every other workgroup starts
 * scoring at once.  Larger pages take the two launches (the append is too long a chain of loads to hide inside
 * the scoring kernel).  cache->seq_lens holds the lengths
 * BEFORE the append (slot n_b is written) and is not modified; the scores cover n_b + 1 tokens, so add 1 to
 * every entry before the selection and decode calls.  Arguments as in the two calls it replaces; both
 * statistics arrays must be given whatever `mode` scores. */
ekv_status ekv_append_score_pages(const ekv_config* cfg, const ekv_cache_view* cache,
                                  const ekv_stats_view* stats, const void* k_new, const void* v_new,
                                  const void* q, int32_t mode, float* box, float* mu, float* sigma,
                                  void* stream);

/* a5 -- fixed-budget top-k page selection (Sec. 4.3).  For each (b,h): the min(k_pages, M_b) pages
 * of largest box score among p < M_b; equal scores (-0 and +0 are equal) are resolved towards the lower page index.
 * page_idx int32 [B][Hq][cap] receives the logical page indices in ASCENDING order, n_sel int32
 * [B][Hq] their number.  Requires 1 <= k_pages <= cap and a workspace of
 * ekv_workspace_bytes(EKV_OP_SELECT_TOPK) bytes (long contexts are split over several workgroups per
 * head, which exchange histograms through it). */
ekv_status ekv_select_topk(const ekv_config* cfg, const float* box, const int32_t* seq_lens,
                           int32_t k_pages, int32_t* page_idx, int32_t* n_sel, void* workspace,
                           size_t workspace_bytes, void* stream);

/* a6 -- Gaussian-aware selector (Sec. 4.3 Eq. 10-12, App. D).  Per (b,h): solves
 *   sum_{p<M_b} cnt_p E[(a S_p - tau)_+^beta] = 1,  S_p ~ N(mu_p, sigma_p^2)      (Eq. 10)
 * for tau_hat (closed-form truncated Gaussian moments, iterated to float32 convergence), then keeps
 * page p iff a*(mu_p + sigma_p * PhiInv(q_page^(1/cnt_p))) > tau_hat - margin       (Eq. 11-12).
 * An empty result is replaced by the single best page; more than cap pages keeps the cap pages of
 * largest estimate (lower index first on ties) and sets overflow[b,h]=1 (else 0).
 * tau_hat f32 [B][Hq]; page_idx/n_sel as in ekv_select_topk; overflow int32 [B][Hq].
 * Range: alpha with integer 1/(alpha-1) in 1..4 and max_pages_per_seq <= 4 194 304, else EKV_ERR_UNSUPPORTED.
 * 0 < q_page < 1, margin >= 0.  beta must be 1, 2, 3 or 4. */
ekv_status ekv_select_gauss(const ekv_config* cfg, const float* mu, const float* sigma,
                            const int32_t* seq_lens, float q_page, float margin, float* tau_hat,
                            int32_t* page_idx, int32_t* n_sel, int32_t* overflow, void* workspace,
                            size_t workspace_bytes, void* stream);

/* Box-threshold selection and refinement (App. B.2: with a threshold that does not exceed the exact one,
 * the page bounds of Eq. 9 never miss a page that holds a support token).  Per (b,h):
 *   page_idx_out = page_idx_in[0..n_sel_in)  UNION  { p < M_b : a * box[b,h,p] > tau_lo[b,h] },  ascending,
 * n_sel_out its size, n_added the pages of the second set that were not in the first.
 * Use: tau_lo := tau of ekv_decode_sparse over page_idx_in (a sparse threshold never exceeds the
 * full-cache one).  n_added == 0 certifies that sparse result as exact; otherwise the output list holds
 * the whole support and one more ekv_decode_sparse over it is exact (Sec. 3.2, exact recovery).
 * box f32 [B][Hq][Mmax] from ekv_score_pages; tau_lo f32 [B][Hq] (device; +inf selects nothing, -inf
 * every page); page_idx_in/n_sel_in may both be NULL (empty list; entries outside [0, M_b) are ignored,
 * order and duplicates do not matter); page_idx_out int32 [B][Hq][cap] may alias page_idx_in, n_sel_out
 * may alias n_sel_in; n_added, overflow int32 [B][Hq].  If the union exceeds cap, its first cap pages (by
 * index) are written and overflow[b,h]=1: the list is then incomplete and certifies nothing.
 * Workspace: ekv_workspace_bytes(EKV_OP_SELECT_BOX_THRESHOLD).  Range: max_pages_per_seq <= 4 194 304 (else
 * EKV_ERR_UNSUPPORTED, also from ekv_workspace_bytes). */
ekv_status ekv_select_box_threshold(const ekv_config* cfg, const float* box, const int32_t* seq_lens,
                                    const float* tau_lo, const int32_t* page_idx_in,
                                    const int32_t* n_sel_in, int32_t* page_idx_out, int32_t* n_sel_out,
                                    int32_t* n_added, int32_t* overflow, void* workspace,
                                    size_t workspace_bytes, void* stream);

/* Optional side outputs of the decode calls (all device pointers, any may be NULL).
 *   support_tokens int32 [B][Hq][support_cap]: logical token indices j with p_j > 0, in candidate
 *       order (ascending when page_idx is ascending); only the first support_cap are written.
 *   tau_ref f32 [B][Hq] (input): a reference threshold (normally the full-cache tau); when given,
 *       kept_mass_ref[b,h] = sum_{j in candidates} (z_j - tau_ref)_+^beta   (1 - dropped mass, Eq. 4)
 *       kept_supp_ref[b,h] = #{j in candidates : z_j > tau_ref}             (numerator of Eq. 7)
 *   lse f32 [B][Hq] (ekv_decode_full only): log sum_j exp(scale q.k_j) over the whole cache.
 *   tau_seed f32 [B][Hq] (input): a guess of tau for a warm start -- the Gaussian-aware estimate
 *       tau-hat of the same query (Sec. 4.3 uses it as the solver's starting point), or the threshold
 *       of an earlier solve.  It only chooses where the exact solve starts: the first evaluation is taken
 *       at the seed when it lies inside the certified bracket, and, on rows of at most 262 144 candidates,
 *       a seed that the group maxima certify as a lower bound of tau also serves as the candidate
 *       threshold.  Any value (wrong, infinite, NaN) is safe; tau, supp and out do not depend on it
 *       beyond float32 rounding of the last iterate.
 *   solve_evals int32 [B][Hq]: number of evaluations of the mass sum_j (z_j - tau)_+^beta the solve
 *       took (a measure of what a seed saves).
 *   score_pass_only: measurement aid.  Non-zero: only the first pass runs (gather of the K pages, scores and group
 *       maxima into the workspace); out, tau, supp and every other output are left untouched.  It lets the
 *       HBM-bound kernel of the decode be timed on its own. */
typedef struct {
  int32_t* support_tokens;
  int32_t support_cap;
  const float* tau_ref;
  float* kept_mass_ref;
  int32_t* kept_supp_ref;
  float* lse;
  const float* tau_seed;
  int32_t* solve_evals;
  int32_t score_pass_only;
} ekv_decode_extras;

/* a7 -- sparse alpha-entmax attention over the selected pages (Sec. 4.1, Sec. 4.4).
 * Candidates of (b,h): tokens j < n_b of the pages page_idx[b,h,0..n_sel[b,h]).  z_j = a*scale*q.k_j;
 * tau is the EXACT root of sum_j (z_j - tau)_+^beta = 1 over the candidates (float32 arithmetic);
 * p_j = (z_j - tau)_+^beta; out = sum_j p_j v_j.  V rows are read only where p_j > 0.
 * out f32 [B][Hq][d]; tau f32 [B][Hq]; supp int32 [B][Hq] = #{j: z_j > tau}.  extras may be NULL. */
ekv_status ekv_decode_sparse(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                             const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                             int32_t* supp, const ekv_decode_extras* extras, void* workspace,
                             size_t workspace_bytes, void* stream);

/* For callers that cannot allocate device memory and have no workspace to pass (code recorded into a HIP graph,
 * tight serving loops, harnesses that forbid hipMalloc): ekv_decode_sparse with the same arguments, results and
 * kernels, but with its scratch in a static device array inside the library instead of a caller workspace.  The call
 * allocates nothing and frees nothing.  The array has EKV_STATIC_SCRATCH_BYTES bytes; a configuration whose
 * ekv_workspace_bytes(cfg, EKV_OP_DECODE_SPARSE, ..) exceeds that is rejected with EKV_ERR_WORKSPACE before anything
 * is launched.  Each GPU the library runs on holds its own copy of the array until the process ends, and every call on
 * a GPU uses that one copy: calls that overlap in time on one GPU (different streams or threads) race on it and must
 * be serialised by the caller; calls in one stream are safe.  Nothing in the array has to start at zero (every value
 * a kernel reads is written earlier in the same call), so a call does not depend on what the previous one left.
 * Other errors as ekv_decode_sparse; EKV_ERR_HIP if the array's device address cannot be obtained. */
#define EKV_STATIC_SCRATCH_BYTES (32u << 20)
ekv_status ekv_decode_sparse_static(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                                    const int32_t* page_idx, const int32_t* n_sel, float* out, float* tau,
                                    int32_t* supp, const ekv_decode_extras* extras, void* stream);

/* a7, page lists shared per KV head: as ekv_decode_sparse, but page_idx int32 [B][Hkv][cap] and n_sel
 * int32 [B][Hkv] hold one list per KV head and every query head of the group attends over it (its own
 * tau, support and output).  K of a selected page is read once for the whole group (a [G x d] x [d x P]
 * tile on the matrix cores), i.e. 1/G of the per-head gather.  Outputs, extras and workspace
 * (EKV_OP_DECODE_SPARSE) are those of ekv_decode_sparse. */
ekv_status ekv_decode_sparse_group(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                                   const int32_t* page_idx, const int32_t* n_sel, float* out,
                                   float* tau, int32_t* supp, const ekv_decode_extras* extras,
                                   void* workspace, size_t workspace_bytes, void* stream);

/* a8 -- dense full-cache alpha-entmax decode (Sec. 2.1 Eq. 1 with pi = entmax): ekv_decode_sparse
 * with every page p < M_b selected.  K is streamed once per KV head for its G query heads. */
ekv_status ekv_decode_full(const ekv_config* cfg, const void* q, const ekv_cache_view* cache,
                           float* out, float* tau, int32_t* supp, const ekv_decode_extras* extras,
                           void* workspace, size_t workspace_bytes, void* stream);

/* a9 -- softmax attention restricted to the same selected pages (the sparse softmax baseline of
 * Sec. 5.5 / App. E.1), with its kept mass against the full-cache normaliser (Eq. 8):
 * out f32 [B][Hq][d] = sum_j softmax(scale q.k_j over candidates) v_j; lse_sel f32 [B][Hq] = log-sum-exp
 * over the candidates (so kept softmax mass = exp(lse_sel - lse_full)). */
ekv_status ekv_decode_sparse_softmax(const ekv_config* cfg, const void* q,
                                     const ekv_cache_view* cache, const int32_t* page_idx,
                                     const int32_t* n_sel, float* out, float* lse_sel,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Measurement aid, no part of the method: reads n_pages pages of page_bytes bytes (4096 or 8192) of the device
 * buffer `base` and discards the data, four pages per wavefront.  Page i of the launch is page page_ids[i] of the
 * buffer (device int32 list), or page lookup[page_ids[i]] when `lookup` (device int32 table) is given -- a second
 * dependent read per page, as the decode does through page list and block table.  Every resulting page number must
 * lie inside the buffer; it is NOT checked.  With a permutation the probe has the access pattern of the sparse
 * decode's gather, with the identity that of a linear stream: the rate it reaches is the ceiling a read-only kernel
 * gets on the GPU at hand, reported next to the published HBM peak.  `out` (optional, device float
 * [ceil(n_pages/4) * 64]): every wavefront also writes 256 bytes, the output volume of the decode's score pass.
 * `sink`: 4 bytes of device memory (written only in a practically impossible case).  Asynchronous on `stream`;
 * EKV_ERR_INVALID_ARG for null or misaligned pointers or n_pages <= 0, EKV_ERR_UNSUPPORTED for other page sizes. */
ekv_status ekv_probe_read(const void* base, const int32_t* page_ids, const int32_t* lookup, int32_t n_pages,
                          int32_t page_bytes, float* out, void* sink, void* stream);

/* Measurement aid, no part of the method: what handing data from workgroup to workgroup inside ONE launch costs on
 * the GPU at hand, compared with a kernel boundary -- the question behind every "fuse these two dependent stages"
 * idea.  n_workgroups (2..65536) workgroups write 4 KiB each into `data` (device float [n_workgroups * 1024]); mode 0:
 * nothing more; mode 1: device-scope fence + acquire-release counter, the last workgroup to arrive fences and reads
 * 8 KiB written by others; mode 2: no fences, device-scope atomic (write-through) stores, relaxed counter, atomic
 * loads by the last arriver.  `counter`: device uint32, zero before the first call (each launch leaves it at zero);
 * `out`: device float, receives a checksum (accumulated).  Asynchronous on `stream`. */
ekv_status ekv_probe_handoff(float* data, uint32_t* counter, float* out, int32_t n_workgroups, int32_t mode,
                             void* stream);

/* Bytes of workspace `op` needs under cfg (host computation, no HIP calls). */
ekv_status ekv_workspace_bytes(const ekv_config* cfg, int32_t op, size_t* bytes);

/* Name of a status code (static string). */
const char* ekv_status_string(int32_t status);

/* hipError_t code of the most recent failing HIP call on this thread (0 if none). */
int32_t ekv_last_hip_error(void);

/* Library version, e.g. 100 for 0.1.0. */
int32_t ekv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ENTMAXKV_H */
