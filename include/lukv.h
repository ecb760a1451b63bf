/*
 * lukv.h - C ABI of the LU-KV prefill-time KV-cache eviction path for AMD MI355X (gfx950).
 *
 * The path (paper: "Predicting Future Utility: Global Combinatorial Optimization for
 * Task-Agnostic KV Cache Eviction"):
 *   score    observation-window attention metric per KV head           (Eq. 1; SnapKV, App. D)
 *   allocate global head-level budgets on the convex-hull relaxation    (Sec. 4.2, Eq. 8-10, App. A.2)
 *   select   per-head top-b_{l,h} positions by the metric               (Sec. 3.2 M^pi(k); Sec. 4.3 "Eviction")
 *   compact  the retained index sets as a dense per-head cache          (Sec. 3.2, Eq. 3)
 * and, around it: the score with the window rows' log-sum-exp supplied (Sec. 4.3), the offline
 * profile and its online look-up (Sec. 4.1 Eq. 6, Sec. 4.3 Eq. 11), and a decode step's
 * attention over the compacted cache (Eq. 3).
 *
 * Conventions common to every call
 *   - "device" pointers are GPU memory owned by the caller (any allocator); "host" pointers are
 *     ordinary process memory read during the call only.  The library never allocates, frees or
 *     keeps a pointer.  Its only scratch is the caller's workspace `ws` of at least
 *     lukv_workspace_bytes() bytes, 256-byte aligned; contents need not be initialised and are
 *     clobbered.  Two calls that share a workspace must not overlap in time.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work; they never synchronise the host and never copy to or from the host.
 *   - Results are deterministic: the same inputs give bitwise the same outputs.
 *   - Return value: LUKV_OK (0) = enqueued; negative = refused on the host, nothing enqueued
 *     and no output touched.  Conditions only visible on the device are reported through the
 *     device `status` words.  No C++ exception crosses the boundary.
 *   - Head order everywhere: flat head index hi = (seq * n_layers + layer) * n_kv_heads + kv_head.
 *     Sequences are packed along the token axis; sequence s owns tokens
 *     [cu_seqlens[s], cu_seqlens[s+1]) and window-query rows [s*window, (s+1)*window).
 *   - Limits: 1 <= n_seqs <= LUKV_MAX_SEQS; head_dim in {64, 128}; (n_q_heads/n_kv_heads)*window
 *     <= 512 (<= 256 for f32 with head_dim 128); pool_kernel odd, 1..31; every sequence longer
 *     than `window`, at most 1 048 576 tokens long, and n_sink <= L - window; at most 2^31-1
 *     packed tokens; one sequence's keys of one head span less than 4 GiB
 *     (L * stride_tok * element size < 2^32).
 */
#ifndef LUKV_H
#define LUKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LUKV_OK            0
#define LUKV_EINVAL       (-1)  /* null pointer, bad dimension, stride or limit */
#define LUKV_EDTYPE       (-2)  /* unknown dtype / unsupported dtype-head_dim combination */
#define LUKV_EINFEASIBLE  (-3)  /* host-visible infeasible budget (B < 0) */
#define LUKV_EWORKSPACE   (-4)  /* workspace missing, misaligned or too small */
#define LUKV_ELAUNCH      (-5)  /* the HIP runtime refused a launch */

#define LUKV_BF16 0             /* Q, K, V stored as bfloat16 */
#define LUKV_F32  1             /* Q, K, V stored as float32 */

#define LUKV_MAX_SEQS 64

/* device status bits */
#define LUKV_ST_INFEASIBLE 1    /* allocation: B outside [sum b_min, sum min(b_max, L)] */
#define LUKV_ST_CLAMPED    2    /* selection: a budget outside [0, L] was clamped */

typedef struct lukv_config {
  int32_t n_layers;       /* layers in this call */
  int32_t n_q_heads;      /* query heads per layer */
  int32_t n_kv_heads;     /* KV heads per layer; must divide n_q_heads (GQA group G) */
  int32_t head_dim;       /* d_h */
  int32_t window;         /* observation window w: the last w queries of each sequence */
  int32_t pool_kernel;    /* 1-D max-pool width p (odd), stride 1, clipped at both ends */
  int32_t n_sink;         /* first n_sink positions of a sequence are always kept */
  int32_t dtype;          /* LUKV_BF16 | LUKV_F32: storage type of q_win, k, v */
  int32_t n_seqs;         /* packed sequences */
  const int32_t* cu_seqlens; /* HOST [n_seqs+1], cu_seqlens[0] = 0, increasing */
  int64_t stride_layer, stride_head, stride_tok;    /* element strides of k and v:
                             x[layer][kv_head][token][0..d) at layer*sl + head*sh + token*st;
                             the d elements of a row are contiguous; rows 16-byte aligned */
  int64_t qstride_layer, qstride_head, qstride_tok; /* element strides of q_win:
                             q_win[layer][q_head][seq*window + i][0..d) */
  float softmax_scale;    /* 0 => 1/sqrt(head_dim) (Eq. 1) */
} lukv_config;

/* Bytes of workspace any call below needs for this configuration (host only, pure).
 * n_grid = grid points per utility curve (0 if lukv_allocate / lukv_evict are not used). */
int lukv_workspace_bytes(const lukv_config* cfg, int32_t n_grid, int64_t* bytes);

/* Bytes of workspace a stand-alone lukv_allocate call needs (never more than
 * lukv_workspace_bytes for a configuration with the same heads and n_grid). */
int lukv_allocate_workspace_bytes(int32_t n_problems, int32_t n_heads, int32_t n_grid,
                                  int64_t* bytes);

/* Step 1, Eq. 1 + SnapKV metric (App. D Table 8: window 32, kernel 7).
 * For every KV head: softmax(q.k/sqrt(d)) of each window query over the keys it can see
 * (window row i of a length-L sequence sits at position L-w+i and sees keys 0..L-w+i), summed
 * over the w rows, averaged over the G query heads of the group, max-pooled over the prefix
 * [0, L-w); positions >= L-w and < n_sink are set to +inf (always kept, App. E).
 *   q_win  device, dtype, strides qstride_*        k  device, dtype, strides stride_*
 *   pooled device float32 [n_layers][n_kv_heads][total_tokens], written in full. */
int lukv_score(const lukv_config* cfg, const void* q_win, const void* k, float* pooled,
               void* ws, int64_t ws_bytes, void* stream);

/* Step 2, Sec. 4.2 / App. A.2: n_problems independent allocations (one per sequence), each over
 * n_heads heads.  Per head the utility curve (knots[g], curves[g]) is replaced by its upper
 * concave hull (the PAVA surrogate of Eq. 9); every head first gets b_min; the remaining
 * B - sum(b_min) units go to the largest marginal gains over all heads (equal gains: lowest
 * head, then lowest unit), never beyond min(b_max, last knot).  Gains are compared as
 * (double(U_b) - double(U_a)) / double(n_b - n_a), IEEE, no fused multiply-add.
 *   curves  device float32 [n_problems][n_heads][n_grid], finite
 *   knots   device int32   [n_problems][n_heads][n_grid], knots[..][0] = 0, strictly increasing
 *   b_min, b_max device int32 [n_problems][n_heads]
 *   B_total HOST int64 [n_problems]
 *   budgets device int32 [n_problems*n_heads]      (sum over a problem = B_total when feasible)
 *   offsets device int64 [n_problems*n_heads + 1]  exclusive prefix sum of budgets
 *   status  device int32 [n_problems]: 0, or LUKV_ST_INFEASIBLE (then budgets = b_min)
 * Limits: n_problems <= LUKV_MAX_SEQS, 2 <= n_grid <= 1980. */
int lukv_allocate(int32_t n_problems, int32_t n_heads, int32_t n_grid,
                  const float* curves, const int32_t* knots,
                  const int32_t* b_min, const int32_t* b_max, const int64_t* B_total,
                  int32_t* budgets, int64_t* offsets, int32_t* status,
                  void* ws, int64_t ws_bytes, void* stream);

/* Alternative to lukv_allocate: the baseline allocation Sec. 4.2's opening and Sec. 5.1
 * "Baselines" describe (global top-k over surrogate scores).  Per sequence the positions of all
 * n_heads = n_layers * n_kv_heads heads are pooled and the B_total[s] of largest pooled score are
 * retained; budgets[s][h] is the number of positions of head h among them.  The pooled order is
 * score descending, then head ascending, then position ascending - the selection's tie rule
 * extended by the head index - so lukv_select_compact with these budgets retains exactly that
 * set.  b_floor >= 0 is a safeguard: every head first keeps its b_floor best positions, and the
 * other B_total - n_heads * b_floor places go to the best of all remaining candidates.
 *   pooled  device float32 [n_layers][n_kv_heads][total_tokens] as lukv_score writes it
 *           (+inf = always kept); NaN is not allowed
 *   B_total HOST int64 [n_seqs]
 *   budgets device int32 [n_seqs][n_heads]     offsets device int64 [n_seqs * n_heads + 1]
 *   status  device int32 [n_seqs]: 0, or LUKV_ST_INFEASIBLE when b_floor > L, B_total <
 *           n_heads * b_floor or B_total > n_heads * L (then budgets = b_floor)
 *   ws: lukv_workspace_bytes(cfg, 0) bytes.  Limit: n_heads <= 4096.
 * The paper compares against this allocation; it gives no kernel for it. */
int lukv_allocate_topk(const lukv_config* cfg, const float* pooled, const int64_t* B_total,
                       int32_t b_floor, int32_t* budgets, int64_t* offsets, int32_t* status,
                       void* ws, int64_t ws_bytes, void* stream);

/* Steps 3+4: per head hi keep the budgets[hi] positions of largest pooled score (ties: lowest
 * position), and gather their K and V rows.
 *   pooled   device float32 [n_layers][n_kv_heads][total_tokens] (no NaN)
 *   budgets  device int32 [n_heads_total], offsets device int64 [n_heads_total+1]
 *   out_rows rows the three outputs hold (normally offsets[n_heads_total]); only rows in
 *            [0, out_rows) are ever written: a row at or beyond out_rows is dropped, a head whose
 *            offsets[hi] is negative writes nothing at all, and LUKV_ST_CLAMPED is raised instead.
 *            Offsets need not be monotone (heads may then overwrite each other's rows)
 *   kept_idx device int32 [out_rows]: kept_idx[offsets[hi] + r] = r-th kept position (within its
 *            sequence, ascending)
 *   k_out, v_out device, dtype, [out_rows][head_dim]: row offsets[hi]+r, contiguous
 *   status   device int32 [1]: 0 or LUKV_ST_CLAMPED (a budget outside [0, L] was clamped, or rows
 *            were dropped for lack of room) */
int lukv_select_compact(const lukv_config* cfg, const float* pooled, const int32_t* budgets,
                        const int64_t* offsets, const void* k, const void* v, int64_t out_rows,
                        int32_t* kept_idx, void* k_out, void* v_out, int32_t* status,
                        void* ws, int64_t ws_bytes, void* stream);

/* The whole path: allocate (one problem per sequence over n_layers*n_kv_heads heads, ordered
 * (layer, kv_head)) -> score -> select -> compact, enqueued back to back.
 * Arguments as above; pooled may be NULL (scores then stay in the workspace).  kept_idx, k_out
 * and v_out hold sum(B_total) rows.
 *   status device int32 [n_seqs + 1]: [s] allocation status of sequence s, [n_seqs] selection.
 * The selection uses every budget clamped to [0, L] (LUKV_ST_CLAMPED if one was outside, which
 * can only happen for an infeasible problem whose b_min is itself out of range), and `offsets`
 * is the prefix sum of the clamped budgets, so no row outside [0, sum(B_total)) is written. */
int lukv_evict(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
               int32_t n_grid, const float* curves, const int32_t* knots,
               const int32_t* b_min, const int32_t* b_max, const int64_t* B_total,
               int32_t* budgets, int64_t* offsets, int32_t* kept_idx,
               void* k_out, void* v_out, float* pooled, int32_t* status,
               void* ws, int64_t ws_bytes, void* stream);

/* Variants of lukv_score and lukv_evict for callers whose prefill attention kernel already
 * leaves the log of Eq. 1's denominator for the window rows (Sec. 4.3: the observation-window
 * scores are a by-product of prefill): the pass over K that recomputes the softmax statistics is
 * skipped and probabilities are exp(scale * q.k - lse).
 *   lse device float32 [n_layers][n_q_heads][n_seqs * window], contiguous: natural log of the sum
 *       over the visible keys (0 .. L-w+i for window row i) of exp(softmax_scale * q.k).
 * Everything else as in lukv_score / lukv_evict.  A wrong lse scales that row's contribution; it
 * is not checked. */
int lukv_score_lse(const lukv_config* cfg, const void* q_win, const void* k, const float* lse,
                   float* pooled, void* ws, int64_t ws_bytes, void* stream);
int lukv_evict_lse(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                   const float* lse, int32_t n_grid, const float* curves, const int32_t* knots,
                   const int32_t* b_min, const int32_t* b_max, const int64_t* B_total,
                   int32_t* budgets, int64_t* offsets, int32_t* kept_idx,
                   void* k_out, void* v_out, float* pooled, int32_t* status,
                   void* ws, int64_t ws_bytes, void* stream);

/* The static profile and the online look-up (Sec. 4.3: Eq. 11 and "Online Execution" steps 1-2).
 *
 * lukv_profile_build: for every calibration query m (its own utility curves, as in
 * lukv_allocate) and every global compression ratio rho[r] of the grid, the relaxed allocation
 * with B = floor((1 - rho[r]) * L * n_heads) gives local ratios 1 - b/L; phi[r][h] is their
 * mean over the queries (fp64 sum in query order, divided by n_queries, rounded to float).  A
 * ratio whose B is infeasible takes lukv_allocate's result for that case (budgets = b_min).
 *   curves, knots device [n_queries][n_heads][n_grid]; b_min, b_max device [n_queries][n_heads]
 *   rho HOST double [n_rho], strictly increasing;  phi device float32 [n_rho][n_heads]
 *   ws: lukv_profile_workspace_bytes(n_queries, n_heads, n_grid) bytes.
 * Limits as lukv_allocate (n_queries <= LUKV_MAX_SEQS), 1 <= n_rho, 1 <= L.
 *
 * lukv_budgets_from_profile: local ratios at sigma_target, linear between the two neighbouring
 * grid ratios (the end rows outside the grid): t = (sigma - rho_i) / (rho_{i+1} - rho_i),
 * r = phi_i + t * (phi_{i+1} - phi_i) in fp64; budgets[h] = floor((1 - r) * L) kept inside
 * [b_min[h], b_max[h]]; offsets = exclusive prefix sum.  Needs no workspace.
 *   phi device [n_rho][n_heads]; b_min, b_max device int32 [n_heads]
 *   budgets device int32 [n_heads]; offsets device int64 [n_heads + 1]. */
int lukv_profile_workspace_bytes(int32_t n_queries, int32_t n_heads, int32_t n_grid, int64_t* bytes);

/* Offline profiling, first step (Sec. 4.1, Eq. 6): the utility curve of a head from per-token
 * importance and the heuristic metric's ranking.  For each of n_curves (query, head) pairs the T
 * tokens are ranked by (score descending, index ascending); U(i) is the importance of the first i
 * tokens of the ranking (fp64 running sum); curves[c][g] = float(U(knots[c][g])).  The result is
 * what lukv_profile_build and lukv_allocate take as `curves`.
 *   importance, scores device float32 [n_curves][T] (importance >= 0, scores without NaN)
 *   knots device int32 [n_curves][n_grid], values in [0, T] (others are clamped)
 *   curves device float32 [n_curves][n_grid]
 * Limits: 1 <= T <= 4096 (one profiled context is sorted in LDS), n_grid >= 1. */
int lukv_profile_curves(int32_t n_curves, int32_t T, int32_t n_grid, const float* importance,
                        const float* scores, const int32_t* knots, float* curves, void* stream);
int lukv_profile_build(int32_t n_queries, int32_t n_heads, int32_t n_grid, const float* curves,
                       const int32_t* knots, const int32_t* b_min, const int32_t* b_max, int32_t L,
                       int32_t n_rho, const double* rho, float* phi, void* ws, int64_t ws_bytes,
                       void* stream);
int lukv_budgets_from_profile(int32_t n_heads, int32_t n_rho, const double* rho, const float* phi,
                              double sigma_target, int32_t L, const int32_t* b_min,
                              const int32_t* b_max, int32_t* budgets, int64_t* offsets, void* stream);

/* The online mode's eviction (Sec. 4.3 "Online Execution" step 3): budgets are given (for
 * example by lukv_budgets_from_profile), so score -> select -> compact run without the
 * allocation.  Heads ordered as everywhere (one sequence's heads are (layer, kv_head)).
 *   lse may be NULL (the statistics pass then runs) or as in lukv_score_lse
 *   budgets device int32 [n_heads_total], offsets device int64 [n_heads_total + 1] (inputs)
 *   out_rows, kept_idx, k_out, v_out, status [1] as in lukv_select_compact; pooled may be NULL. */
int lukv_evict_budgets(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                       const float* lse, const int32_t* budgets, const int64_t* offsets,
                       int64_t out_rows, int32_t* kept_idx, void* k_out, void* v_out, float* pooled,
                       int32_t* status, void* ws, int64_t ws_bytes, void* stream);

/* Consumer of the compacted cache: one decode step's attention over the retained entries of
 * every head (Sec. 3.2, Eq. 3 restricted to the retained index sets).  For head hi and each of
 * the G query heads of its group: out = softmax_r(softmax_scale * q . K_r) V over the packed rows
 * r in [offsets[hi], offsets[hi+1]); zeros for a head without rows.  fp32 accumulation.
 *   cfg      dimensions, dtype, cu_seqlens (for the longest sequence) and softmax_scale as above;
 *            n_q_heads / n_kv_heads <= 16
 *   q_dec    device, dtype, contiguous [n_layers][n_q_heads][n_seqs][head_dim]: one query per
 *            sequence and query head
 *   k_packed, v_packed, offsets as written by lukv_evict / lukv_select_compact
 *   out      device float32, contiguous [n_layers][n_q_heads][n_seqs][head_dim]
 *   ws       lukv_decode_workspace_bytes(cfg) bytes, 256-byte aligned. */
int lukv_decode_workspace_bytes(const lukv_config* cfg, int64_t* bytes);
int lukv_decode_attention(const lukv_config* cfg, const void* q_dec, const void* k_packed,
                          const void* v_packed, const int64_t* offsets, float* out, void* ws,
                          int64_t ws_bytes, void* stream);

/* lukv_evict for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as lukv_evict, but the scratch is a fixed array inside the library
 * (LUKV_STATIC_SCRATCH_BYTES of device memory per GPU the library runs on, held until the process
 * ends); the call allocates and frees nothing.  A configuration whose lukv_workspace_bytes exceeds
 * LUKV_STATIC_SCRATCH_BYTES is refused with LUKV_EWORKSPACE (the 8B-shaped layer at 32k context
 * needs 7.4 MiB).  Every call on a GPU uses that GPU's one array: calls that overlap in time on
 * the same GPU (different streams or threads) race and must be serialised by the caller.  The
 * array needs no clearing between calls (every word is written before it is read in a call). */
#define LUKV_STATIC_SCRATCH_BYTES (16 << 20)
int lukv_evict_static(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                      int32_t n_grid, const float* curves, const int32_t* knots,
                      const int32_t* b_min, const int32_t* b_max, const int64_t* B_total,
                      int32_t* budgets, int64_t* offsets, int32_t* kept_idx,
                      void* k_out, void* v_out, float* pooled, int32_t* status, void* stream);

/* Static description of a return code. */
const char* lukv_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LUKV_H */
