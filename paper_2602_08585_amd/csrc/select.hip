// Steps 3 and 4: per-head top-b_{l,h} by the metric (Sec. 3.2, M^pi(k); Sec. 4.3 "Eviction")
// with the fixed tie rule App. A.1 assumes (lowest position first), and the gather of the
// retained rows into a dense per-head cache (Sec. 3.2, Eq. 3).
//
// Exact radix select on order-preserving 32-bit keys, digits of 11, 11 and 10 bits.
//   sel_hist - one workgroup (1024 threads) per slice of 1024 scores: [optionally the clipped
//              max-pool + forced +inf of step 1,] an LDS histogram of the top digit, stored
//              as the slice's own 16-bit counts (no shared hot counters).
//   sel_tail - one workgroup per head: sums the slice histograms, fixes digit 0, re-scans the
//              head's scores for digits 1 and 2, and counts, per block of 256 scores, the
//              keys above and equal to the threshold T (no cross-workgroup counters or
//              fences anywhere: kernel boundaries order the phases).
//   sel_emit - one workgroup per block of 256 scores: prefix over earlier blocks, keep
//              (key > T) plus the first r ties by position, write ascending positions and
//              copy the K and V rows (16 bytes per lane, eight rows in flight per thread).
#include "lukv_internal.hpp"

namespace lukv {

__device__ __forceinline__ unsigned key_of(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;  // -0 and +0 tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct SelGeom {
  int32_t n_layers, n_kv_heads, total_tokens, max_slices, max_blocks;
  int32_t window, pool_kernel, n_sink;
};

// Exclusive scan of one unsigned per thread over 1024 threads; part has 16 slots.
__device__ __forceinline__ unsigned scan1024(unsigned v, unsigned* part) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) part[wave] = incl;
  __syncthreads();
  unsigned before = incl - v;
  for (int w = 0; w < wave; ++w) before += part[w];
  return before;
}

// Slice histogram of the top digit (and, with POOL, the pooled scores themselves).
template <bool POOL>
__global__ __launch_bounds__(1024) void sel_hist_kernel(SelGeom sg, SeqTab tab, const float* src_scores,
                                                        float* pooled_out, unsigned* hist_parts,
                                                        int32_t* status) {
  __shared__ unsigned lh[kHistBins];
  __shared__ float rawt[kSliceElems + 32];
  int seq, sl;
  find_tile(tab, blockIdx.x, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z, t = threadIdx.x;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const int64_t base = ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const float* src = src_scores + base;
  float* pooled = POOL ? pooled_out + base : nullptr;
  unsigned* my_part = hist_parts + ((int64_t)hi * sg.max_slices + sl) * (kHistBins / 2);
  // the selection status word starts at zero; later kernels of the call only OR into it
  if (t == 0 && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) *status = 0;

  lh[t] = 0;
  lh[t + 1024] = 0;
  const int j0 = sl * kSliceElems, j = j0 + t;
  float s = 0.f;
  if (POOL) {
    // clipped max-pool over the prefix [0, P); window and sink positions are forced to +inf
    const int P = L - sg.window, h = sg.pool_kernel >> 1;
    for (int i = t; i < kSliceElems + 2 * h; i += 1024) {
      const int jj = j0 - h + i;
      rawt[i] = (jj >= 0 && jj < P) ? src[jj] : -INFINITY;
    }
    __syncthreads();
    if (j < L) {
      s = INFINITY;
      if (j >= sg.n_sink && j < P) {
        s = rawt[t];
        for (int d = 1; d <= 2 * h; ++d) s = fmaxf(s, rawt[t + d]);
      }
      pooled[j] = s;
    }
  } else {
    __syncthreads();
    if (j < L) s = src[j];
  }
  if (j < L) atomicAdd(&lh[key_of(s) >> 21], 1u);
  __syncthreads();
  my_part[t] = (lh[2 * t] & 0xFFFFu) | (lh[2 * t + 1] << 16);   // counts <= 1024 fit 16 bits
}

// One workgroup per head: fixes the threshold key T and the number of ties to keep,
// state[hi] = {T, ties at T to keep, budget after clamping, 0}, counts per block of 256
// scores, and (if offsets_out is given) this head's row offset = sum of the budgets before it.
__global__ __launch_bounds__(1024) void sel_tail_kernel(SelGeom sg, SeqTab tab, const float* scores,
                                                        const int32_t* budgets, const unsigned* hist_parts,
                                                        uint4* state, uint2* block_cnt,
                                                        int64_t* offsets_out, int n_heads_total,
                                                        int32_t* status) {
  __shared__ unsigned lh[kHistBins];
  __shared__ unsigned part[16];
  __shared__ unsigned sel[2];
  __shared__ long long osum[16];
  const int hi = blockIdx.x, t = threadIdx.x;
  const int kvh = hi % sg.n_kv_heads, layer = (hi / sg.n_kv_heads) % sg.n_layers;
  const int seq = hi / (sg.n_kv_heads * sg.n_layers);
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int n_slices = (L + kSliceElems - 1) / kSliceElems;
  const float* keys_src = scores + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const int lane = t & 63, wave = t >> 6;

  if (offsets_out) {
    long long acc = 0;
    for (int h2 = t; h2 < hi; h2 += 1024) acc += budgets[h2];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const int lo = __shfl_xor((int)(acc & 0xFFFFFFFFll), o), hi32 = __shfl_xor((int)(acc >> 32), o);
      acc += ((long long)hi32 << 32) | (unsigned)lo;
    }
    if (lane == 0) osum[wave] = acc;
    __syncthreads();
    if (t == 0) {
      long long tot = 0;
      for (int w = 0; w < 16; ++w) tot += osum[w];
      offsets_out[hi] = tot;
      if (hi == n_heads_total - 1) offsets_out[n_heads_total] = tot + budgets[hi];
    }
  }

  int kb = budgets[hi];
  if (kb < 0 || kb > L) {
    if (t == 0) atomicOr(status, LUKV_ST_CLAMPED);
    kb = kb < 0 ? 0 : L;
  }
  if (kb == 0) {
    // nothing kept: a threshold above every key and no ties
    if (t == 0) state[hi] = make_uint4(0xFFFFFFFFu, 0u, 0u, 0u);
    const unsigned n_blocks = (L + kEmitElems - 1) / kEmitElems;
    for (unsigned b = t; b < n_blocks; b += 1024) block_cnt[(int64_t)hi * sg.max_blocks + b] = make_uint2(0u, 0u);
    return;
  }
  // digit 0: thread t owns packed word 1023-t, i.e. bins 2047-2t (first) and 2046-2t
  unsigned c_hi = 0, c_lo = 0;
  {
    const unsigned* hp = hist_parts + (int64_t)hi * sg.max_slices * (kHistBins / 2) + (1023 - t);
    for (int s0 = 0; s0 < n_slices; s0 += 8) {
      unsigned w[8];   // independent loads first: one memory latency per eight slices
#pragma unroll
      for (int u = 0; u < 8; ++u) w[u] = s0 + u < n_slices ? hp[(int64_t)(s0 + u) * (kHistBins / 2)] : 0u;
#pragma unroll
      for (int u = 0; u < 8; ++u) { c_lo += w[u] & 0xFFFFu; c_hi += w[u] >> 16; }
    }
  }
  unsigned want = (unsigned)kb, prefix = 0;
  {
    const unsigned before = scan1024(c_hi + c_lo, part);
    if (before < want && want <= before + c_hi) { sel[0] = 2047 - 2 * t; sel[1] = want - before; }
    else if (before + c_hi < want && want <= before + c_hi + c_lo) { sel[0] = 2046 - 2 * t; sel[1] = want - before - c_hi; }
    __syncthreads();
    prefix = sel[0] << 21;
    want = sel[1];
  }
  // digit 1 (bits 20..10) among keys with the same digit 0
  lh[t] = 0;
  lh[t + 1024] = 0;
  __syncthreads();
  for (int jj0 = t; jj0 < L; jj0 += 8 * 1024) {
    float f[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) f[u] = jj0 + u * 1024 < L ? keys_src[jj0 + u * 1024] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned key = key_of(f[u]);
      if (jj0 + u * 1024 < L && (key >> 21) == (prefix >> 21)) atomicAdd(&lh[(key >> 10) & 2047u], 1u);
    }
  }
  __syncthreads();
  {
    const unsigned a1 = lh[2047 - 2 * t], a0 = lh[2046 - 2 * t];
    const unsigned before = scan1024(a1 + a0, part);
    if (before < want && want <= before + a1) { sel[0] = 2047 - 2 * t; sel[1] = want - before; }
    else if (before + a1 < want && want <= before + a1 + a0) { sel[0] = 2046 - 2 * t; sel[1] = want - before - a1; }
    __syncthreads();
    prefix |= sel[0] << 10;
    want = sel[1];
  }
  // digit 2 (bits 9..0)
  __syncthreads();
  lh[t] = 0;
  __syncthreads();
  for (int jj0 = t; jj0 < L; jj0 += 8 * 1024) {
    float f[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) f[u] = jj0 + u * 1024 < L ? keys_src[jj0 + u * 1024] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned key = key_of(f[u]);
      if (jj0 + u * 1024 < L && (key >> 10) == (prefix >> 10)) atomicAdd(&lh[key & 1023u], 1u);
    }
  }
  __syncthreads();
  {
    const unsigned a = lh[1023 - t];
    const unsigned before = scan1024(a, part);
    if (before < want && want <= before + a) { sel[0] = 1023 - t; sel[1] = want - before; }
    __syncthreads();
    prefix |= sel[0];
    want = sel[1];
  }
  const unsigned T = prefix;
  if (t == 0) state[hi] = make_uint4(T, want, (unsigned)kb, 0u);
  // per block of 256 scores: keys above T and keys equal to T (one wave per block)
  const int n_blocks = (L + kEmitElems - 1) / kEmitElems;
  for (int b = wave; b < n_blocks; b += 16) {
    unsigned gt = 0, eq = 0;
    float f[kEmitElems / 64];
#pragma unroll
    for (int i = 0; i < kEmitElems / 64; ++i) {
      const int jj = b * kEmitElems + i * 64 + lane;
      f[i] = jj < L ? keys_src[jj] : 0.f;
    }
#pragma unroll
    for (int i = 0; i < kEmitElems / 64; ++i) {
      const int jj = b * kEmitElems + i * 64 + lane;
      const unsigned key = key_of(f[i]);
      gt += jj < L && key > T;
      eq += jj < L && key == T;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      gt += __shfl_xor(gt, o);
      eq += __shfl_xor(eq, o);
    }
    if (lane == 0) block_cnt[(int64_t)hi * sg.max_blocks + b] = make_uint2(gt, eq);
  }
}

template <int ROW_BYTES>
__global__ __launch_bounds__(256) void sel_emit_kernel(SelGeom sg, SeqTab tab, const float* scores,
                                                       const uint4* state, const uint2* block_cnt,
                                                       const int64_t* offsets, const char* k,
                                                       const char* v, int64_t sl_bytes,
                                                       int64_t sh_bytes, int64_t st_bytes,
                                                       int32_t* kept_idx, char* k_out, char* v_out,
                                                       int64_t out_rows, int32_t* status) {
  __shared__ unsigned red_g[4], red_e[4];
  __shared__ unsigned wkeep[4], weq[4];
  __shared__ int list[kEmitElems];
  int seq, blk;
  find_tile(tab, blockIdx.x, seq, blk);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const float* src = scores + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const uint4 stt = state[hi];
  const unsigned T = stt.x, r_eq = stt.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  const int j = blk * kEmitElems + threadIdx.x;
  const bool in = j < L;
  const unsigned key = in ? key_of(src[j]) : 0u;

  // kept rows in earlier blocks of this head
  unsigned gb = 0, eb = 0;
  for (int s2 = threadIdx.x; s2 < blk; s2 += 256) {
    const uint2 c = block_cnt[(int64_t)hi * sg.max_blocks + s2];
    gb += c.x;
    eb += c.y;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    gb += __shfl_xor(gb, o);
    eb += __shfl_xor(eb, o);
  }
  const bool is_eq = in && key == T;
  const unsigned long long em = __ballot(is_eq);
  if (lane == 0) { red_g[wave] = gb; red_e[wave] = eb; weq[wave] = (unsigned)__popcll(em); }
  __syncthreads();
  const unsigned gt_before = red_g[0] + red_g[1] + red_g[2] + red_g[3];
  const unsigned eq_before = red_e[0] + red_e[1] + red_e[2] + red_e[3];
  const int64_t row0 = offsets[hi] + gt_before + (eq_before < r_eq ? eq_before : r_eq);

  // rank of this tie among the ties of the head, in position order
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  unsigned eq_rank = eq_before + (unsigned)__popcll(em & lt_mask);
  for (int w2 = 0; w2 < wave; ++w2) eq_rank += weq[w2];
  const bool keep = in && (key > T || (is_eq && eq_rank < r_eq));
  const unsigned long long km = __ballot(keep);
  if (lane == 0) wkeep[wave] = (unsigned)__popcll(km);
  __syncthreads();
  unsigned pos = (unsigned)__popcll(km & lt_mask);
  for (int w2 = 0; w2 < wave; ++w2) pos += wkeep[w2];
  unsigned n_keep = wkeep[0] + wkeep[1] + wkeep[2] + wkeep[3];
  if (keep) {
    list[pos] = j;
    if (row0 + pos < out_rows) kept_idx[row0 + pos] = j;
  }
  __syncthreads();

  // rows beyond the caller's capacity are dropped and flagged, never written
  if (row0 + n_keep > out_rows) {
    if (threadIdx.x == 0) atomicOr(status, LUKV_ST_CLAMPED);
    n_keep = row0 < out_rows ? (unsigned)(out_rows - row0) : 0u;
  }
  // gather: 16 bytes per lane, ROW_BYTES/16 lanes per row, four K and four V rows per thread
  constexpr int kLanesPerRow = ROW_BYTES / 16;
  constexpr int kRowsPerIter = 256 / kLanesPerRow;
  constexpr int kUnroll = 4;
  const int rsub = threadIdx.x / kLanesPerRow, col = (threadIdx.x % kLanesPerRow) * 16;
  const char* kb = k + layer * sl_bytes + kvh * sh_bytes + (int64_t)tok0 * st_bytes + col;
  const char* vb = v + layer * sl_bytes + kvh * sh_bytes + (int64_t)tok0 * st_bytes + col;
  char* ko = k_out + row0 * ROW_BYTES + col;
  char* vo = v_out + row0 * ROW_BYTES + col;
  for (unsigned i0 = rsub; i0 < n_keep; i0 += kUnroll * kRowsPerIter) {
    u32x4 kr[kUnroll], vr[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const unsigned i = i0 + u * kRowsPerIter;
      const int jr = list[i < n_keep ? i : i0];
      kr[u] = *reinterpret_cast<const u32x4*>(kb + (int64_t)jr * st_bytes);
      vr[u] = *reinterpret_cast<const u32x4*>(vb + (int64_t)jr * st_bytes);
    }
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const unsigned i = i0 + u * kRowsPerIter;
      if (i < n_keep) {
        *reinterpret_cast<u32x4*>(ko + (int64_t)i * ROW_BYTES) = kr[u];
        *reinterpret_cast<u32x4*>(vo + (int64_t)i * ROW_BYTES) = vr[u];
      }
    }
  }
}

template <int ROW_BYTES>
static void launch_emit(dim3 grid, hipStream_t st, SelGeom sg, const SeqTab& tab, const float* pooled,
                        const uint4* state, const uint2* block_cnt, const int64_t* offsets,
                        const void* k, const void* v, const Geom& g, int esize, int32_t* kept_idx,
                        void* k_out, void* v_out, int64_t out_rows, int32_t* status) {
  hipLaunchKernelGGL((sel_emit_kernel<ROW_BYTES>), grid, dim3(256), 0, st, sg, tab, pooled, state,
                     block_cnt, offsets, (const char*)k, (const char*)v, g.sl * esize, g.sh * esize,
                     g.st * esize, kept_idx, (char*)k_out, (char*)v_out, out_rows, status);
}

// scores_in: pooled scores (pool = false) or the unpooled metric (pool = true; the pooled
// scores are then written to pooled_out and used for the selection).
int launch_select_compact(const HostCfg& hc, const WsLayout& lay, const float* scores_in, bool pool,
                          float* pooled_out, const int32_t* budgets, int64_t* offsets, bool make_offsets,
                          const void* k, const void* v, int32_t* kept_idx, void* k_out, void* v_out,
                          int64_t out_rows, int32_t* status, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  const SeqTab tabH = tiles_for(hc.seq, kSliceElems, 0);
  const SeqTab tabE = tiles_for(hc.seq, kEmitElems, 0);
  SelGeom sg{g.n_layers, g.n_kv_heads, g.total_tokens, lay.max_slices, lay.max_blocks,
             g.window, g.pool_kernel, g.n_sink};
  unsigned* hist = reinterpret_cast<unsigned*>(ws + lay.hist);
  uint4* state = reinterpret_cast<uint4*>(ws + lay.sel_state);
  uint2* block_cnt = reinterpret_cast<uint2*>(ws + lay.slice_cnt);
  dim3 gridH(tabH.tile0[tabH.n_seqs], g.n_kv_heads, g.n_layers);
  dim3 gridE(tabE.tile0[tabE.n_seqs], g.n_kv_heads, g.n_layers);
  stage_mark(kStHist, st);
  if (pool)
    hipLaunchKernelGGL(sel_hist_kernel<true>, gridH, dim3(1024), 0, st, sg, tabH, scores_in, pooled_out,
                       hist, status);
  else
    hipLaunchKernelGGL(sel_hist_kernel<false>, gridH, dim3(1024), 0, st, sg, tabH, scores_in,
                       (float*)nullptr, hist, status);
  const float* sel_scores = pool ? pooled_out : scores_in;
  stage_mark(kStTail, st);
  hipLaunchKernelGGL(sel_tail_kernel, dim3(hc.n_hi), dim3(1024), 0, st, sg, tabH, sel_scores, budgets,
                     (const unsigned*)hist, state, block_cnt, make_offsets ? offsets : (int64_t*)nullptr,
                     hc.n_hi, status);
  stage_mark(kStEmit, st);
  const int esize = g.f32 ? 4 : 2;
  const int row_bytes = g.head_dim * esize;
  if (row_bytes == 128)
    launch_emit<128>(gridE, st, sg, tabE, sel_scores, state, block_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else if (row_bytes == 256)
    launch_emit<256>(gridE, st, sg, tabE, sel_scores, state, block_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else if (row_bytes == 512)
    launch_emit<512>(gridE, st, sg, tabE, sel_scores, state, block_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else
    return LUKV_EDTYPE;
  return check_launch();
}

}  // namespace lukv
