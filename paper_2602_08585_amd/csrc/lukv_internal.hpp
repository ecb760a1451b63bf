// Internal declarations shared by the translation units of liblukv (HIP, gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "lukv.h"

namespace lukv {

// 16 bytes as a first-class vector.  Register arrays must use this, not the uint4 struct:
// arrays of the struct type are not promoted to registers and end up in scratch memory.
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// ---- tiling constants -------------------------------------------------------------------
constexpr int kSliceElems = 1024;  // scores one workgroup of the selection histogram owns
constexpr int kHistBins = 2048;    // bins of the widest radix digit (11 bits)
constexpr int kMaxSeqLen = 1 << 20;  // tokens per sequence (1024 slices: one selection thread per slice)
constexpr int kMaxGrid = 1980;     // utility-curve grid points (hull stack lives in LDS)
constexpr int kMaxRows = 512;      // G * window upper bound

// Packed-sequence table passed to kernels by value: sequence boundaries plus the first tile
// of every sequence for the tile size of the launch.
struct SeqTab {
  int32_t n_seqs;
  int32_t cu[LUKV_MAX_SEQS + 1];     // token offsets
  int32_t tile0[LUKV_MAX_SEQS + 1];  // tile offsets (prefix sum of tiles per sequence)
};

// Geometry of a call, by value to every kernel.
struct Geom {
  int32_t n_layers, n_q_heads, n_kv_heads, group, head_dim;
  int32_t window, pool_kernel, n_sink, f32;
  int32_t rows;        // G * window
  int32_t row_blocks;  // ceil(rows / 32)
  int32_t row_groups;  // 1, 2 or 4 wave groups share the row blocks
  int32_t blocks_per_group;
  int32_t total_tokens;
  int32_t chunk_keys;  // keys one workgroup of the score kernels streams (multiple of 128)
  int64_t sl, sh, st;     // K/V strides (elements)
  int64_t qsl, qsh, qst;  // Q strides (elements)
  float scale_log2e;      // softmax scale * log2(e)
  float inv_group;        // 1 / G
};

// Byte offsets into the caller's workspace.
struct WsLayout {
  int64_t alloc_vertex;          // i32 [n_problems * n_heads * n_grid]
  int64_t hist;                  // u32 [n_hi * max_slices * kHistBins / 2] packed 16-bit suffix counts
  int64_t range;                 // float2 [n_hi * range_stride] (min, max) of the metric per chunk part
  int64_t head_dig;              // uint2 [n_hi] first digit of the selection: (base key, shift)
  int64_t by_bin;                // u64 [n_layers * n_kv_heads * total_tokens] (key, position) by slice and bin
  int64_t cand;                  // u64, same shape: threshold candidates of a head beyond the LDS list
  int64_t partial;               // float [n_hi * 64 * rows_padded] log-sum of every (granule of keys, row)
  int64_t raw;                   // float [n_layers * n_kv_heads * total_tokens]
  int64_t pooled;                // float, same shape
  int64_t sel_state;             // uint4 [n_hi]
  int64_t slice_cnt;             // uint2 [n_hi * max_slices] kept rows / ties before each slice
  int64_t seg_key;               // u64 [n_problems * n_heads * n_grid]
  int64_t seg_w;                 // u32 [n_problems * n_heads * n_grid]
  int64_t keepmask;              // u32 [n_hi * 1024] whole-head selection: keep bits of every 32-position run
  int64_t runpre;                // u32 [n_hi * 1032] kept rows before every run (entry 1024: the head's total)
  int64_t head_flag;             // u32 [n_hi] status bits a head raised
  int64_t topk;                  // scratch of the global top-k allocation
  int64_t total;
  int32_t n_hi, max_chunks, max_slices, range_stride, rows_padded;
};

struct HostCfg {
  Geom g;
  SeqTab seq;       // cu filled, tile0 unset
  int32_t max_len;  // longest sequence
  int32_t n_hi;
};

int validate_config(const lukv_config* cfg, HostCfg* out);
WsLayout make_layout(const HostCfg& hc, int32_t n_grid, bool alloc_only);
SeqTab tiles_for(const SeqTab& seq, int tile, int shrink);  // tiles over (L_s - shrink) tokens

// Launchers (enqueue only; return a LUKV_* code).
struct AllocIO;
// raw (unpooled) metric into the workspace; aio != NULL: the allocation's first phase (hull
// vertices) rides along in the score kernels
// lse != NULL: the window rows' log-sum-exp is given, pass A is not launched
int launch_score_raw(const HostCfg& hc, const WsLayout& lay, const void* q, const void* k,
                     const float* lse, const AllocIO* aio, char* ws, hipStream_t st);
int launch_pool(const HostCfg& hc, const WsLayout& lay, float* pooled_out, char* ws, hipStream_t st);
// aio != NULL: the allocation's second phase rides along in the first selection kernel
int launch_select_compact(const HostCfg& hc, const WsLayout& lay, const AllocIO* aio,
                          const float* scores_in, bool pool,
                          float* pooled_out, const int32_t* budgets, int64_t* offsets,
                          bool make_offsets, const void* k, const void* v, int32_t* kept_idx, void* k_out, void* v_out,
                          int64_t out_rows, int32_t* status, char* ws, hipStream_t st);
// every sequence short enough for the whole-head form of the selection (scores of a head in LDS)
bool select_whole_head(const HostCfg& hc);
AllocIO make_alloc_io(int32_t n_problems, int32_t n_heads, int32_t n_grid, const float* curves,
                      const int32_t* knots, const int32_t* b_min, const int32_t* b_max,
                      const int64_t* B_total, int32_t* budgets, int64_t* offsets, int32_t* status,
                      const WsLayout& lay, char* ws);
int launch_allocate(const AllocIO& io, hipStream_t st);
void launch_allocate_budgets(const AllocIO& io, hipStream_t st);    // second phase only (no offsets)
void launch_offsets(const int32_t* budgets, int64_t* offsets, int64_t n_all, hipStream_t st);   // prefix sum
// baseline allocation by a global top-k over pooled scores (topk_alloc.hip); ws points at its
// own scratch of topk_workspace_bytes
int64_t topk_workspace_bytes(int32_t n_seqs, int32_t n_heads);
int launch_allocate_topk(const HostCfg& hc, const float* scores, const int64_t* B_total, int32_t floor,
                         int32_t* budgets, int64_t* offsets, int32_t* status, char* ws, hipStream_t st);
// static profile (Eq. 11): io0 describes the calibration queries as allocation problems whose
// budgets / status arrays are scratch; rho is a host array
int launch_profile_build(const AllocIO& io0, int32_t L, int32_t n_rho, const double* rho, float* phi,
                         hipStream_t st);
int launch_profile_lookup(const float* row_lo, const float* row_hi, double t, int32_t n_heads, int32_t L,
                          const int32_t* b_min, const int32_t* b_max, int32_t* budgets, int64_t* offsets,
                          hipStream_t st);

// utility curves from per-token importance (profile.hip)
int launch_profile_curves(int32_t n_curves, int32_t T, int32_t n_grid, const float* importance,
                          const float* scores, const int32_t* knots, float* curves, hipStream_t st);

// decode-step attention over the packed cache (decode.hip)
int64_t decode_workspace_bytes(const HostCfg& hc);
int launch_decode(const HostCfg& hc, const void* q, const void* kp, const void* vp, const int64_t* offsets,
                  float* out, char* ws, hipStream_t st);

// Optional instrumentation (lukv_set_stage_events): the main kernel of a stage is launched with
// the caller's start / stop events attached to its own dispatch.
enum Stage { kStAllocate = 0, kStStats, kStAccum, kStPool, kStHist, kStTail, kStEmit, kStHead, kStGather, kNumStages };
void stage_events(int stage, hipEvent_t* start, hipEvent_t* stop);   // NULLs when none are set

template <class... KArgs, class... Args>
inline void launch_staged(int stage, void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t st,
                          Args... args) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  stage_events(stage, &e0, &e1);
  if (e0 || e1)
    hipExtLaunchKernelGGL(kernel, grid, block, 0, st, e0, e1, 0, static_cast<KArgs>(args)...);
  else
    hipLaunchKernelGGL(kernel, grid, block, 0, st, static_cast<KArgs>(args)...);
}

inline int check_launch() {
  return hipGetLastError() == hipSuccess ? LUKV_OK : LUKV_ELAUNCH;
}

// Sequence / tile lookup for a flat tile index (linear scan, n_seqs <= 64, wave-uniform).
__device__ inline void find_tile(const SeqTab& tab, int tile, int& seq, int& local_tile) {
  int s = 0;
  while (s + 1 < tab.n_seqs && tile >= tab.tile0[s + 1]) ++s;
  seq = s;
  local_tile = tile - tab.tile0[s];
}

// Inclusive scan over the 64 lanes of a wave with DPP row shifts and row broadcasts (no LDS
// crossbar traffic): four shifts scan each row of 16 lanes, lane 15 of rows 0 and 2 is then
// broadcast into rows 1 and 3, and lane 31 into rows 2 and 3.
__device__ __forceinline__ unsigned wave_scan_incl(unsigned v) {
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, true);   // row_shr:1
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, true);   // row_shr:2
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, true);   // row_shr:4
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, true);   // row_shr:8
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false);  // row_bcast:15
  v += (unsigned)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false);  // row_bcast:31
  return v;
}

// Reductions over the 64 lanes of a wave with the same DPP steps; the result is valid in lane 63.
// `ident` is the operation's identity (what a lane without a source contributes).
template <class Op>
__device__ __forceinline__ unsigned wave_reduce_to_last(unsigned v, unsigned ident, Op op) {
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x111, 0xf, 0xf, false));
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x112, 0xf, 0xf, false));
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x114, 0xf, 0xf, false));
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x118, 0xf, 0xf, false));
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x142, 0xa, 0xf, false));
  v = op(v, (unsigned)__builtin_amdgcn_update_dpp((int)ident, (int)v, 0x143, 0xc, 0xf, false));
  return v;
}

// Exclusive scan of one unsigned per thread over the workgroup (<= 16 waves); part has 16 slots.
// Every thread of the workgroup calls it (two barriers inside).  The wave totals are scanned
// by every wave for itself (one LDS read per lane, no serial chain over the waves).
__device__ __forceinline__ unsigned block_scan_u32(unsigned v, unsigned* part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  const unsigned incl = wave_scan_incl(v);
  __syncthreads();
  if (lane == 63) part[wave] = incl;
  __syncthreads();
  const unsigned tot = lane < n_waves ? part[lane] : 0u;
  const unsigned upto = wave_scan_incl(tot);
  const unsigned before_wave = (unsigned)__builtin_amdgcn_readlane((int)(upto - tot), wave);
  return before_wave + incl - v;
}

}  // namespace lukv
