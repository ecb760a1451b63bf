// C ABI of liblukv: argument checks, workspace layout, and the order of launches.
#include <math.h>
#include <string.h>

#include <mutex>

#include "alloc_device.hpp"
#include "lukv_internal.hpp"

// Scratch of lukv_evict_static: one array per GPU, inside the library's code object.  In host
// code the name below is only a handle for hipGetSymbolAddress; kernels and launches get the
// device address that call returned for the current device (static_scratch_ptr).
static __device__ __align__(256) unsigned char scratch[LUKV_STATIC_SCRATCH_BYTES];

namespace lukv {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on every device seen so far

// Device address of the static scratch on the current device (asked once per device, with that
// device current); nullptr when the runtime refuses.  Allocates nothing.
static void* static_scratch_ptr() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

static inline int64_t align_up(int64_t x, int64_t a) { return (x + a - 1) / a * a; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate_config(const lukv_config* cfg, HostCfg* out) {
  if (!cfg || !out || !cfg->cu_seqlens) return LUKV_EINVAL;
  if (cfg->dtype != LUKV_BF16 && cfg->dtype != LUKV_F32) return LUKV_EDTYPE;
  if (cfg->head_dim != 64 && cfg->head_dim != 128) return LUKV_EDTYPE;
  if (cfg->n_layers < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1) return LUKV_EINVAL;
  if (cfg->n_layers > 65535 || cfg->n_kv_heads > 65535) return LUKV_EINVAL;
  if (cfg->n_q_heads % cfg->n_kv_heads) return LUKV_EINVAL;
  if (cfg->window < 1 || cfg->n_sink < 0) return LUKV_EINVAL;
  if (cfg->pool_kernel < 1 || cfg->pool_kernel > 31 || !(cfg->pool_kernel & 1)) return LUKV_EINVAL;
  if (cfg->n_seqs < 1 || cfg->n_seqs > LUKV_MAX_SEQS) return LUKV_EINVAL;
  if (!(cfg->softmax_scale >= 0.f) || isinf(cfg->softmax_scale)) return LUKV_EINVAL;
  const int esize = cfg->dtype == LUKV_F32 ? 4 : 2;
  const int64_t strides[6] = {cfg->stride_layer, cfg->stride_head, cfg->stride_tok,
                              cfg->qstride_layer, cfg->qstride_head, cfg->qstride_tok};
  for (int i = 0; i < 6; ++i)
    if (strides[i] < 0 || (strides[i] * esize) % 16) return LUKV_EINVAL;
  if (cfg->stride_tok < cfg->head_dim || cfg->qstride_tok < cfg->head_dim) return LUKV_EINVAL;

  Geom& g = out->g;
  memset(out, 0, sizeof(*out));
  g.n_layers = cfg->n_layers;
  g.n_q_heads = cfg->n_q_heads;
  g.n_kv_heads = cfg->n_kv_heads;
  g.group = cfg->n_q_heads / cfg->n_kv_heads;
  g.head_dim = cfg->head_dim;
  g.window = cfg->window;
  g.pool_kernel = cfg->pool_kernel;
  g.n_sink = cfg->n_sink;
  g.f32 = cfg->dtype == LUKV_F32;
  const int64_t rows = (int64_t)g.group * g.window;
  const int nbm = (g.f32 && g.head_dim == 128) ? 2 : 4;
  if (rows > 128 * nbm) return LUKV_EINVAL;
  g.rows = (int32_t)rows;
  g.row_blocks = (g.rows + 31) / 32;
  g.row_groups = g.row_blocks <= nbm ? 1 : (g.row_blocks <= 2 * nbm ? 2 : 4);
  g.blocks_per_group = (g.row_blocks + g.row_groups - 1) / g.row_groups;
  g.sl = cfg->stride_layer; g.sh = cfg->stride_head; g.st = cfg->stride_tok;
  g.qsl = cfg->qstride_layer; g.qsh = cfg->qstride_head; g.qst = cfg->qstride_tok;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / sqrtf((float)g.head_dim);
  g.scale_log2e = scale * 1.4426950408889634f;
  g.inv_group = 1.0f / (float)g.group;

  out->seq.n_seqs = cfg->n_seqs;
  if (cfg->cu_seqlens[0] != 0) return LUKV_EINVAL;
  int32_t max_len = 0;
  for (int s = 0; s < cfg->n_seqs; ++s) {
    const int64_t a = cfg->cu_seqlens[s], b = cfg->cu_seqlens[s + 1];
    const int64_t L = b - a;
    if (L <= g.window || g.n_sink > L - g.window || L > kMaxSeqLen) return LUKV_EINVAL;
    out->seq.cu[s] = (int32_t)a;
    out->seq.cu[s + 1] = (int32_t)b;
    if (L > max_len) max_len = (int32_t)L;
  }
  g.total_tokens = out->seq.cu[cfg->n_seqs];
  // the kernels address one head's keys of one sequence with 32-bit byte offsets
  if ((int64_t)max_len * cfg->stride_tok * esize >= (1ll << 32)) return LUKV_EINVAL;
  out->max_len = max_len;
  // Keys per score workgroup: a multiple of every sequence's granule of softmax statistics (512
  // keys, doubled until the sequence has at most 64 granules).  Calls with many workgroups
  // (several layers, long batches) take longer chunks: the prologue of a score workgroup (queries,
  // first tile, merge of the granules' statistics) is then paid once per 1024 or 2048 keys.  The
  // thresholds are in units of the 512 workgroups a 256-unit chip holds at once, from timings at
  // 1 to 32 layers of 32k context; they are constants, so that the chunking - which never
  // changes a result - is a function of the configuration alone.
  g.chunk_keys = 512;
  while ((max_len + g.chunk_keys - 1) / g.chunk_keys > 64) g.chunk_keys *= 2;
  {
    auto n_wgs = [&](int chunk) {
      int64_t n = 0;
      for (int s = 0; s < cfg->n_seqs; ++s) n += (out->seq.cu[s + 1] - out->seq.cu[s] + chunk - 1) / chunk;
      return n * g.n_kv_heads * g.n_layers;
    };
    if (g.chunk_keys < 1024 && n_wgs(1024) >= 1024) g.chunk_keys = 1024;
    if (g.chunk_keys == 1024 && n_wgs(2048) >= 2048) g.chunk_keys = 2048;
  }
  out->n_hi = cfg->n_seqs * g.n_layers * g.n_kv_heads;
  return LUKV_OK;
}

SeqTab tiles_for(const SeqTab& seq, int tile, int shrink) {
  SeqTab t = seq;
  t.tile0[0] = 0;
  for (int s = 0; s < seq.n_seqs; ++s) {
    const int len = seq.cu[s + 1] - seq.cu[s] - shrink;
    t.tile0[s + 1] = t.tile0[s] + (len + tile - 1) / tile;
  }
  return t;
}

WsLayout make_layout(const HostCfg& hc, int32_t n_grid, bool alloc_only) {
  WsLayout w;
  memset(&w, 0, sizeof(w));
  const Geom& g = hc.g;
  w.n_hi = hc.n_hi;
  w.max_chunks = g.chunk_keys > 0 ? (hc.max_len + g.chunk_keys - 1) / g.chunk_keys : 0;
  w.max_slices = (hc.max_len + kSliceElems - 1) / kSliceElems;
  w.range_stride = w.max_chunks * 4 > w.max_slices ? w.max_chunks * 4 : w.max_slices;
  w.rows_padded = g.row_blocks * 32;
  int64_t off = 0;
  auto take = [&](int64_t bytes) { const int64_t o = off; off = align_up(off + bytes, 256); return o; };
  const int64_t n_sel = alloc_only ? 0 : w.n_hi;
  w.hist = take(n_sel * w.max_slices * (kHistBins / 2) * 4);
  w.partial = take((int64_t)w.n_hi * 64 * w.rows_padded * 4);   // one log-sum per (granule of keys, row)
  const int64_t score_bytes = (int64_t)g.n_layers * g.n_kv_heads * g.total_tokens * 4;
  w.raw = take(score_bytes);
  w.pooled = take(score_bytes);
  w.sel_state = take(n_sel * 16);
  w.slice_cnt = take(n_sel * w.max_slices * 8);
  w.range = take(n_sel * w.range_stride * 8);
  w.head_dig = take(n_sel * 8);
  w.by_bin = take(alloc_only ? 0 : score_bytes * 2);
  w.cand = take(alloc_only ? 0 : score_bytes * 2);
  const int64_t nseg = (int64_t)hc.n_hi * (n_grid > 0 ? n_grid : 0);
  w.alloc_vertex = take(nseg * 4);
  w.seg_key = take(nseg * 8);
  w.seg_w = take(nseg * 4);
  w.keepmask = take(n_sel * 1024 * 4);
  w.runpre = take(n_sel * 1032 * 4);
  w.head_flag = take(n_sel * 4);
  w.topk = take(alloc_only ? 0 : topk_workspace_bytes(hc.seq.n_seqs, hc.g.n_layers * hc.g.n_kv_heads));
  w.total = off;
  return w;
}

static int check_ws(const WsLayout& lay, const void* ws, int64_t ws_bytes) {
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < lay.total) return LUKV_EWORKSPACE;
  return LUKV_OK;
}

// Layout for a stand-alone lukv_allocate call (no lukv_config).
static WsLayout alloc_only_layout(int32_t n_problems, int32_t n_heads, int32_t n_grid) {
  HostCfg hc;
  memset(&hc, 0, sizeof(hc));
  hc.n_hi = n_problems * n_heads;
  hc.max_len = 0;
  return make_layout(hc, n_grid, true);
}

}  // namespace lukv

using namespace lukv;

extern "C" {

int lukv_workspace_bytes(const lukv_config* cfg, int32_t n_grid, int64_t* bytes) {
  if (!bytes || n_grid < 0 || n_grid > kMaxGrid) return LUKV_EINVAL;
  HostCfg hc;
  const int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  *bytes = make_layout(hc, n_grid, false).total;
  return LUKV_OK;
}

int lukv_allocate_workspace_bytes(int32_t n_problems, int32_t n_heads, int32_t n_grid,
                                  int64_t* bytes) {
  if (!bytes || n_problems < 1 || n_problems > LUKV_MAX_SEQS || n_heads < 1 || n_grid < 2 ||
      n_grid > kMaxGrid)
    return LUKV_EINVAL;
  if ((int64_t)n_problems * n_heads > (1 << 24)) return LUKV_EINVAL;
  *bytes = alloc_only_layout(n_problems, n_heads, n_grid).total;
  return LUKV_OK;
}

static int score_impl(const lukv_config* cfg, const void* q_win, const void* k, const float* lse,
                      float* pooled, void* ws, int64_t ws_bytes, void* stream) {
  HostCfg hc;
  int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (!q_win || !k || !pooled || !aligned16(q_win) || !aligned16(k)) return LUKV_EINVAL;
  const WsLayout lay = make_layout(hc, 0, false);
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = launch_score_raw(hc, lay, q_win, k, lse, nullptr, (char*)ws, st))) return rc;
  return launch_pool(hc, lay, pooled, (char*)ws, st);
}

int lukv_score(const lukv_config* cfg, const void* q_win, const void* k, float* pooled,
               void* ws, int64_t ws_bytes, void* stream) {
  return score_impl(cfg, q_win, k, nullptr, pooled, ws, ws_bytes, stream);
}

int lukv_score_lse(const lukv_config* cfg, const void* q_win, const void* k, const float* lse,
                   float* pooled, void* ws, int64_t ws_bytes, void* stream) {
  if (!lse) return LUKV_EINVAL;
  return score_impl(cfg, q_win, k, lse, pooled, ws, ws_bytes, stream);
}

int lukv_allocate(int32_t n_problems, int32_t n_heads, int32_t n_grid, const float* curves,
                  const int32_t* knots, const int32_t* b_min, const int32_t* b_max,
                  const int64_t* B_total, int32_t* budgets, int64_t* offsets, int32_t* status,
                  void* ws, int64_t ws_bytes, void* stream) {
  if (n_problems < 1 || n_problems > LUKV_MAX_SEQS || n_heads < 1 || n_grid < 2 || n_grid > kMaxGrid)
    return LUKV_EINVAL;
  if ((int64_t)n_problems * n_heads > (1 << 24)) return LUKV_EINVAL;
  if (!curves || !knots || !b_min || !b_max || !B_total || !budgets || !offsets || !status)
    return LUKV_EINVAL;
  for (int i = 0; i < n_problems; ++i)
    if (B_total[i] < 0) return LUKV_EINFEASIBLE;
  // the allocation scratch sits at the same offsets as in a full configuration with the
  // same number of heads only when there is no score/select scratch before it, so a
  // stand-alone call lays the workspace out on its own
  const WsLayout lay = alloc_only_layout(n_problems, n_heads, n_grid);
  int rc;
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  return launch_allocate(make_alloc_io(n_problems, n_heads, n_grid, curves, knots, b_min, b_max, B_total,
                                       budgets, offsets, status, lay, (char*)ws), st);
}

int lukv_allocate_topk(const lukv_config* cfg, const float* pooled, const int64_t* B_total, int32_t b_floor,
                       int32_t* budgets, int64_t* offsets, int32_t* status, void* ws, int64_t ws_bytes,
                       void* stream) {
  HostCfg hc;
  int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (!pooled || !B_total || !budgets || !offsets || !status || b_floor < 0) return LUKV_EINVAL;
  for (int i = 0; i < hc.seq.n_seqs; ++i)
    if (B_total[i] < 0) return LUKV_EINFEASIBLE;
  const WsLayout lay = make_layout(hc, 0, false);
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  return launch_allocate_topk(hc, pooled, B_total, b_floor, budgets, offsets, status, (char*)ws + lay.topk,
                              static_cast<hipStream_t>(stream));
}

int lukv_select_compact(const lukv_config* cfg, const float* pooled, const int32_t* budgets,
                        const int64_t* offsets, const void* k, const void* v, int64_t out_rows,
                        int32_t* kept_idx, void* k_out, void* v_out, int32_t* status, void* ws,
                        int64_t ws_bytes, void* stream) {
  HostCfg hc;
  int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (!pooled || !budgets || !offsets || !k || !v || !kept_idx || !k_out || !v_out || !status)
    return LUKV_EINVAL;
  if (out_rows < 0) return LUKV_EINVAL;
  if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out)) return LUKV_EINVAL;
  const WsLayout lay = make_layout(hc, 0, false);
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  return launch_select_compact(hc, lay, nullptr, pooled, false, nullptr, budgets, const_cast<int64_t*>(offsets),
                               false, k, v, kept_idx, k_out, v_out, out_rows, status, (char*)ws, st);
}

static int evict_impl(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
               const float* lse,
               int32_t n_grid, const float* curves, const int32_t* knots, const int32_t* b_min,
               const int32_t* b_max, const int64_t* B_total, int32_t* budgets, int64_t* offsets,
               int32_t* kept_idx, void* k_out, void* v_out, float* pooled, int32_t* status,
               void* ws, int64_t ws_bytes, void* stream) {
  HostCfg hc;
  int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (n_grid < 2 || n_grid > kMaxGrid) return LUKV_EINVAL;
  if (!q_win || !k || !v || !curves || !knots || !b_min || !b_max || !B_total || !budgets ||
      !offsets || !kept_idx || !k_out || !v_out || !status)
    return LUKV_EINVAL;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
    return LUKV_EINVAL;
  int64_t out_rows = 0;
  for (int i = 0; i < cfg->n_seqs; ++i) {
    if (B_total[i] < 0) return LUKV_EINFEASIBLE;
    out_rows += B_total[i];
  }
  const WsLayout lay = make_layout(hc, n_grid, false);
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = (char*)ws;
  // the whole-head selection keeps the pooled scores in registers: they are only written out when
  // the caller asks for them
  float* scores = pooled ? pooled : (select_whole_head(hc) ? nullptr : reinterpret_cast<float*>(w + lay.pooled));
  int32_t* sel_status = status + cfg->n_seqs;
  // the allocation never looks at scores: its first phase rides along in the score kernels, its
  // second with the selection or between the two; selection pools the raw metric on the fly
  const int n_heads = hc.g.n_layers * hc.g.n_kv_heads;
  const AllocIO aio = make_alloc_io(cfg->n_seqs, n_heads, n_grid, curves, knots, b_min, b_max, B_total,
                                    budgets, offsets, status, lay, w);
  // Where the budget phase runs: with the whole-head selection, inside the head workgroups when
  // the call holds one small allocation problem, else in a launch of its own ahead of them (one
  // workgroup per problem); with the per-slice selection, as extra workgroups of its first kernel.
  const bool whole = select_whole_head(hc);
  const bool b_in_head = whole && cfg->n_seqs == 1 && alloc_small_ok(n_heads, n_grid);
  const bool b_alone = whole && !b_in_head;
  if ((rc = launch_score_raw(hc, lay, q_win, k, lse, &aio, w, st))) return rc;
  if (b_alone) launch_allocate_budgets(aio, st);
  rc = launch_select_compact(hc, lay, b_alone ? nullptr : &aio, reinterpret_cast<const float*>(w + lay.raw), true,
                             scores, budgets, offsets, true, k, v, kept_idx, k_out, v_out, out_rows, sel_status,
                             w, st);
  return rc;
}

int lukv_evict(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
               int32_t n_grid, const float* curves, const int32_t* knots, const int32_t* b_min,
               const int32_t* b_max, const int64_t* B_total, int32_t* budgets, int64_t* offsets,
               int32_t* kept_idx, void* k_out, void* v_out, float* pooled, int32_t* status,
               void* ws, int64_t ws_bytes, void* stream) {
  return evict_impl(cfg, q_win, k, v, nullptr, n_grid, curves, knots, b_min, b_max, B_total, budgets,
                    offsets, kept_idx, k_out, v_out, pooled, status, ws, ws_bytes, stream);
}

int lukv_evict_static(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                      int32_t n_grid, const float* curves, const int32_t* knots, const int32_t* b_min,
                      const int32_t* b_max, const int64_t* B_total, int32_t* budgets, int64_t* offsets,
                      int32_t* kept_idx, void* k_out, void* v_out, float* pooled, int32_t* status,
                      void* stream) {
  // the size check comes first and touches no device: a configuration beyond the built-in
  // scratch is refused before anything else happens
  if (n_grid < 2 || n_grid > kMaxGrid) return LUKV_EINVAL;
  HostCfg hc;
  const int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (make_layout(hc, n_grid, false).total > (int64_t)LUKV_STATIC_SCRATCH_BYTES) return LUKV_EWORKSPACE;
  void* ptr = static_scratch_ptr();
  if (!ptr) return LUKV_ELAUNCH;
  return evict_impl(cfg, q_win, k, v, nullptr, n_grid, curves, knots, b_min, b_max, B_total, budgets,
                    offsets, kept_idx, k_out, v_out, pooled, status, ptr, LUKV_STATIC_SCRATCH_BYTES, stream);
}

int lukv_evict_lse(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                   const float* lse, int32_t n_grid, const float* curves, const int32_t* knots,
                   const int32_t* b_min, const int32_t* b_max, const int64_t* B_total,
                   int32_t* budgets, int64_t* offsets, int32_t* kept_idx, void* k_out, void* v_out,
                   float* pooled, int32_t* status, void* ws, int64_t ws_bytes, void* stream) {
  if (!lse) return LUKV_EINVAL;
  return evict_impl(cfg, q_win, k, v, lse, n_grid, curves, knots, b_min, b_max, B_total, budgets,
                    offsets, kept_idx, k_out, v_out, pooled, status, ws, ws_bytes, stream);
}

// profile scratch after the allocation scratch: budgets, offsets, status of the queries
struct ProfileWs { WsLayout lay; int64_t budgets, offsets, status, total; };
static ProfileWs profile_layout(int32_t n_queries, int32_t n_heads, int32_t n_grid) {
  ProfileWs p;
  p.lay = alloc_only_layout(n_queries, n_heads, n_grid);
  int64_t off = p.lay.total;
  auto take = [&](int64_t bytes) { const int64_t o = off; off = align_up(off + bytes, 256); return o; };
  p.budgets = take((int64_t)n_queries * n_heads * 4);
  p.offsets = take(((int64_t)n_queries * n_heads + 1) * 8);
  p.status = take((int64_t)n_queries * 4);
  p.total = off;
  return p;
}

static bool profile_dims_ok(int32_t n_queries, int32_t n_heads, int32_t n_grid) {
  return n_queries >= 1 && n_queries <= LUKV_MAX_SEQS && n_heads >= 1 && n_grid >= 2 && n_grid <= kMaxGrid &&
         (int64_t)n_queries * n_heads <= (1 << 24);
}

int lukv_profile_workspace_bytes(int32_t n_queries, int32_t n_heads, int32_t n_grid, int64_t* bytes) {
  if (!bytes || !profile_dims_ok(n_queries, n_heads, n_grid)) return LUKV_EINVAL;
  *bytes = profile_layout(n_queries, n_heads, n_grid).total;
  return LUKV_OK;
}

int lukv_profile_curves(int32_t n_curves, int32_t T, int32_t n_grid, const float* importance,
                        const float* scores, const int32_t* knots, float* curves, void* stream) {
  if (n_curves < 1 || T < 1 || T > 4096 || n_grid < 1 || !importance || !scores || !knots || !curves)
    return LUKV_EINVAL;
  return launch_profile_curves(n_curves, T, n_grid, importance, scores, knots, curves,
                               static_cast<hipStream_t>(stream));
}

int lukv_profile_build(int32_t n_queries, int32_t n_heads, int32_t n_grid, const float* curves,
                       const int32_t* knots, const int32_t* b_min, const int32_t* b_max, int32_t L,
                       int32_t n_rho, const double* rho, float* phi, void* ws, int64_t ws_bytes,
                       void* stream) {
  if (!profile_dims_ok(n_queries, n_heads, n_grid) || L < 1 || n_rho < 1) return LUKV_EINVAL;
  if (!curves || !knots || !b_min || !b_max || !rho || !phi) return LUKV_EINVAL;
  for (int r = 0; r < n_rho; ++r)
    if (!(rho[r] == rho[r]) || (r > 0 && !(rho[r] > rho[r - 1]))) return LUKV_EINVAL;
  const ProfileWs pw = profile_layout(n_queries, n_heads, n_grid);
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < pw.total) return LUKV_EWORKSPACE;
  char* w = (char*)ws;
  const AllocIO io = make_alloc_io(n_queries, n_heads, n_grid, curves, knots, b_min, b_max, nullptr,
                                   reinterpret_cast<int32_t*>(w + pw.budgets),
                                   reinterpret_cast<int64_t*>(w + pw.offsets),
                                   reinterpret_cast<int32_t*>(w + pw.status), pw.lay, w);
  return launch_profile_build(io, L, n_rho, rho, phi, static_cast<hipStream_t>(stream));
}

int lukv_budgets_from_profile(int32_t n_heads, int32_t n_rho, const double* rho, const float* phi,
                              double sigma_target, int32_t L, const int32_t* b_min,
                              const int32_t* b_max, int32_t* budgets, int64_t* offsets, void* stream) {
  if (n_heads < 1 || n_rho < 1 || L < 1 || !rho || !phi || !b_min || !b_max || !budgets || !offsets)
    return LUKV_EINVAL;
  if (!(sigma_target == sigma_target)) return LUKV_EINVAL;
  for (int r = 1; r < n_rho; ++r)
    if (!(rho[r] > rho[r - 1])) return LUKV_EINVAL;
  int lo = 0, hi = 0;
  double t = 0.0;
  if (n_rho == 1 || sigma_target <= rho[0]) {
    lo = hi = 0;
  } else if (sigma_target >= rho[n_rho - 1]) {
    lo = hi = n_rho - 1;
  } else {
    for (int r = 0; r + 1 < n_rho; ++r)
      if (rho[r] <= sigma_target) lo = r;
    hi = lo + 1;
    t = (sigma_target - rho[lo]) / (rho[hi] - rho[lo]);
  }
  return launch_profile_lookup(phi + (int64_t)lo * n_heads, phi + (int64_t)hi * n_heads, t, n_heads, L, b_min,
                               b_max, budgets, offsets, static_cast<hipStream_t>(stream));
}

int lukv_evict_budgets(const lukv_config* cfg, const void* q_win, const void* k, const void* v,
                       const float* lse, const int32_t* budgets, const int64_t* offsets,
                       int64_t out_rows, int32_t* kept_idx, void* k_out, void* v_out, float* pooled,
                       int32_t* status, void* ws, int64_t ws_bytes, void* stream) {
  HostCfg hc;
  int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (!q_win || !k || !v || !budgets || !offsets || !kept_idx || !k_out || !v_out || !status || out_rows < 0)
    return LUKV_EINVAL;
  if (!aligned16(q_win) || !aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out))
    return LUKV_EINVAL;
  const WsLayout lay = make_layout(hc, 0, false);
  if ((rc = check_ws(lay, ws, ws_bytes))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* w = (char*)ws;
  float* scores = pooled ? pooled : (select_whole_head(hc) ? nullptr : reinterpret_cast<float*>(w + lay.pooled));
  if ((rc = launch_score_raw(hc, lay, q_win, k, lse, nullptr, w, st))) return rc;
  rc = launch_select_compact(hc, lay, nullptr, reinterpret_cast<const float*>(w + lay.raw), true, scores, budgets,
                             const_cast<int64_t*>(offsets), false, k, v, kept_idx, k_out, v_out, out_rows,
                             status, w, st);
  return rc;
}

int lukv_decode_workspace_bytes(const lukv_config* cfg, int64_t* bytes) {
  if (!bytes) return LUKV_EINVAL;
  HostCfg hc;
  const int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (hc.g.group > 16) return LUKV_EINVAL;
  *bytes = align_up(decode_workspace_bytes(hc), 256);
  return LUKV_OK;
}

int lukv_decode_attention(const lukv_config* cfg, const void* q_dec, const void* k_packed,
                          const void* v_packed, const int64_t* offsets, float* out, void* ws,
                          int64_t ws_bytes, void* stream) {
  HostCfg hc;
  const int rc = validate_config(cfg, &hc);
  if (rc) return rc;
  if (hc.g.group > 16) return LUKV_EINVAL;
  if (!q_dec || !k_packed || !v_packed || !offsets || !out) return LUKV_EINVAL;
  if (!aligned16(k_packed) || !aligned16(v_packed) || !aligned16(q_dec)) return LUKV_EINVAL;
  if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || ws_bytes < decode_workspace_bytes(hc))
    return LUKV_EWORKSPACE;
  return launch_decode(hc, q_dec, k_packed, v_packed, offsets, out, (char*)ws, static_cast<hipStream_t>(stream));
}

const char* lukv_strerror(int code) {
  switch (code) {
    case LUKV_OK: return "ok";
    case LUKV_EINVAL: return "invalid argument (null pointer, dimension, stride, alignment or limit)";
    case LUKV_EDTYPE: return "unsupported dtype or head_dim";
    case LUKV_EINFEASIBLE: return "infeasible budget";
    case LUKV_EWORKSPACE: return "workspace missing, misaligned or too small (or the configuration needs more than the built-in scratch of lukv_evict_static)";
    case LUKV_ELAUNCH: return "HIP launch failed";
    default: return "unknown lukv error code";
  }
}

}  // extern "C"
