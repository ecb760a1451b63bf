// Steps 3 and 4: per-head top-b_{l,h} by the metric (Sec. 3.2, M^pi(k); Sec. 4.3 "Eviction")
// with the fixed tie rule App. A.1 assumes (lowest position first), and the gather of the
// retained rows into a dense per-head cache (Sec. 3.2, Eq. 3).
//
// Exact radix select on order-preserving 32-bit keys, three digits (11, 11, 10 bits), every
// head split into slices of 1024 scores so that the whole chip works on it:
//   hist<p>  - slice histogram of digit p among the keys that match the digits found so far,
//              merged into the head's histogram; the last slice of a head to arrive walks
//              the bins from the top and fixes digit p of the threshold key T.
//   count    - per slice: #keys > T and #keys == T.
//   emit     - per slice: prefix over earlier slices, keep (key > T) plus the first r ties by
//              position, write ascending positions and copy the K and V rows.
#include "lukv_internal.hpp"

namespace lukv {

__device__ __forceinline__ unsigned key_of(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;  // -0 and +0 tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ int digit_shift(int pass) { return pass == 0 ? 21 : (pass == 1 ? 10 : 0); }
__device__ __forceinline__ int digit_bins(int pass) { return pass == 2 ? 1024 : 2048; }

struct SelGeom {
  int32_t n_layers, n_kv_heads, total_tokens, max_slices;
};

// state[hi] = {T prefix, ties (or rank) still to take, clamped budget, 0}
template <int PASS>
__global__ __launch_bounds__(256) void sel_hist_kernel(SelGeom sg, SeqTab tab, const float* pooled,
                                                       const int32_t* budgets, unsigned* hist,
                                                       unsigned* counter, uint4* state,
                                                       int32_t* status) {
  __shared__ unsigned lh[kHistBins];
  __shared__ unsigned wsum[4];
  __shared__ int is_last;
  int seq, sl;
  find_tile(tab, blockIdx.x, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const int n_slices = tab.tile0[seq + 1] - tab.tile0[seq];
  const float* src = pooled + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  constexpr int kShift = PASS == 0 ? 21 : (PASS == 1 ? 10 : 0);
  constexpr int kBins = PASS == 2 ? 1024 : 2048;
  unsigned* gh = hist + ((int64_t)hi * kRadixPasses + PASS) * kHistBins;

  for (int b = threadIdx.x; b < kBins; b += 256) lh[b] = 0;
  unsigned prefix = 0;
  if (PASS > 0) prefix = state[hi].x;
  __syncthreads();
  const int j0 = sl * kSliceElems;
#pragma unroll
  for (int i = 0; i < kSliceElems / 256; ++i) {
    const int j = j0 + i * 256 + threadIdx.x;
    if (j < L) {
      const unsigned key = key_of(src[j]);
      bool match = true;
      if (PASS == 1) match = (key >> 21) == (prefix >> 21);
      if (PASS == 2) match = (key >> 10) == (prefix >> 10);
      if (match) atomicAdd(&lh[(key >> kShift) & (kBins - 1)], 1u);
    }
  }
  __syncthreads();
  for (int b = threadIdx.x; b < kBins; b += 256) {
    const unsigned c = lh[b];
    if (c) atomicAdd(&gh[b], c);
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0)
    is_last = atomicAdd(&counter[hi * 4 + PASS], 1u) == (unsigned)(n_slices - 1);
  __syncthreads();
  if (!is_last) return;
  __threadfence();

  // walk the bins from the largest digit down; thread t owns 'descending' bins [per*t, per*t+per)
  unsigned want, ktot = 0;
  if (PASS == 0) {
    int kb = budgets[hi];
    if (kb < 0 || kb > L) {
      if (threadIdx.x == 0) atomicOr(status, LUKV_ST_CLAMPED);
      kb = kb < 0 ? 0 : L;
    }
    want = ktot = (unsigned)kb;
  } else {
    const uint4 s = state[hi];
    want = s.y;
    ktot = s.z;
  }
  constexpr int kPer = kBins / 256;
  unsigned mine[kPer], tsum = 0;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    mine[i] = __builtin_nontemporal_load(&gh[kBins - 1 - (threadIdx.x * kPer + i)]);
    tsum += mine[i];
  }
  // exclusive scan of tsum over the 256 threads
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned incl = tsum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  if (lane == 63) wsum[wave] = incl;
  __syncthreads();
  unsigned before = incl - tsum;
  for (int w2 = 0; w2 < wave; ++w2) before += wsum[w2];
  if (want == 0) {
    // nothing to keep: threshold above every key, no ties taken
    if (threadIdx.x == 0) state[hi] = make_uint4(0xFFFFFFFFu, 0u, ktot, 0u);
    return;
  }
  unsigned cum = before;
#pragma unroll
  for (int i = 0; i < kPer; ++i) {
    if (cum < want && want <= cum + mine[i]) {
      const unsigned bin = kBins - 1 - (threadIdx.x * kPer + i);
      state[hi] = make_uint4(prefix | (bin << kShift), want - cum, ktot, 0u);
    }
    cum += mine[i];
  }
}

__global__ __launch_bounds__(256) void sel_count_kernel(SelGeom sg, SeqTab tab, const float* pooled,
                                                        const uint4* state, uint2* slice_cnt) {
  __shared__ unsigned wg[4], we[4];
  int seq, sl;
  find_tile(tab, blockIdx.x, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const float* src = pooled + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const unsigned T = state[hi].x;
  unsigned gt = 0, eq = 0;
  const int j0 = sl * kSliceElems;
#pragma unroll
  for (int i = 0; i < kSliceElems / 256; ++i) {
    const int j = j0 + i * 256 + threadIdx.x;
    if (j < L) {
      const unsigned key = key_of(src[j]);
      gt += key > T;
      eq += key == T;
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    gt += __shfl_xor(gt, o);
    eq += __shfl_xor(eq, o);
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) { wg[wave] = gt; we[wave] = eq; }
  __syncthreads();
  if (threadIdx.x == 0)
    slice_cnt[(int64_t)hi * sg.max_slices + sl] =
        make_uint2(wg[0] + wg[1] + wg[2] + wg[3], we[0] + we[1] + we[2] + we[3]);
}

template <int ROW_BYTES>
__global__ __launch_bounds__(256) void sel_emit_kernel(SelGeom sg, SeqTab tab, const float* pooled,
                                                       const uint4* state, const uint2* slice_cnt,
                                                       const int64_t* offsets, const char* k,
                                                       const char* v, int64_t sl_bytes,
                                                       int64_t sh_bytes, int64_t st_bytes,
                                                       int32_t* kept_idx, char* k_out, char* v_out,
                                                       int64_t out_rows, int32_t* status) {
  __shared__ unsigned red_g[4], red_e[4];
  __shared__ unsigned wkeep[4], weq[4];
  __shared__ int list[kSliceElems];
  int seq, sl;
  find_tile(tab, blockIdx.x, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const float* src = pooled + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const uint4 stt = state[hi];
  const unsigned T = stt.x, r_eq = stt.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

  // kept rows in earlier slices of this head
  unsigned gb = 0, eb = 0;
  for (int s2 = threadIdx.x; s2 < sl; s2 += 256) {
    const uint2 c = slice_cnt[(int64_t)hi * sg.max_slices + s2];
    gb += c.x;
    eb += c.y;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    gb += __shfl_xor(gb, o);
    eb += __shfl_xor(eb, o);
  }
  if (lane == 0) { red_g[wave] = gb; red_e[wave] = eb; }
  __syncthreads();
  const unsigned gt_before = red_g[0] + red_g[1] + red_g[2] + red_g[3];
  unsigned eq_seen = red_e[0] + red_e[1] + red_e[2] + red_e[3];
  unsigned n_keep = 0;  // kept so far in this slice
  const int64_t row0 = offsets[hi] + gt_before + (eq_seen < r_eq ? eq_seen : r_eq);

  const int j0 = sl * kSliceElems;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (int i = 0; i < kSliceElems / 256; ++i) {
    const int j = j0 + i * 256 + threadIdx.x;
    unsigned key = 0;
    const bool in = j < L;
    if (in) key = key_of(src[j]);
    const bool is_eq = in && key == T;
    // rank of this tie among the ties of the head, in position order
    const unsigned long long em = __ballot(is_eq);
    if (lane == 0) weq[wave] = (unsigned)__popcll(em);
    __syncthreads();
    unsigned eq_rank = eq_seen + (unsigned)__popcll(em & lt_mask);
    for (int w2 = 0; w2 < wave; ++w2) eq_rank += weq[w2];
    const unsigned eq_round = weq[0] + weq[1] + weq[2] + weq[3];
    const bool keep = in && (key > T || (is_eq && eq_rank < r_eq));
    const unsigned long long km = __ballot(keep);
    if (lane == 0) wkeep[wave] = (unsigned)__popcll(km);
    __syncthreads();
    unsigned pos = n_keep + (unsigned)__popcll(km & lt_mask);
    for (int w2 = 0; w2 < wave; ++w2) pos += wkeep[w2];
    if (keep) {
      list[pos] = j;
      if (row0 + pos < out_rows) kept_idx[row0 + pos] = j;
    }
    n_keep += wkeep[0] + wkeep[1] + wkeep[2] + wkeep[3];
    eq_seen += eq_round;
    __syncthreads();
  }

  // rows beyond the caller's capacity are dropped and flagged, never written
  if (row0 + n_keep > out_rows) {
    if (threadIdx.x == 0) atomicOr(status, LUKV_ST_CLAMPED);
    n_keep = row0 < out_rows ? (unsigned)(out_rows - row0) : 0u;
  }
  // gather: 16 bytes per lane, ROW_BYTES/16 lanes per row
  constexpr int kLanesPerRow = ROW_BYTES / 16;
  constexpr int kRowsPerIter = 256 / kLanesPerRow;
  const int rsub = threadIdx.x / kLanesPerRow, col = (threadIdx.x % kLanesPerRow) * 16;
  const char* kb = k + layer * sl_bytes + kvh * sh_bytes + (int64_t)tok0 * st_bytes;
  const char* vb = v + layer * sl_bytes + kvh * sh_bytes + (int64_t)tok0 * st_bytes;
  for (unsigned i = rsub; i < n_keep; i += 2 * kRowsPerIter) {
    const unsigned i2 = i + kRowsPerIter;
    const int ja = list[i];
    const int jb = i2 < n_keep ? list[i2] : ja;
    const uint4 ka = *reinterpret_cast<const uint4*>(kb + (int64_t)ja * st_bytes + col);
    const uint4 va = *reinterpret_cast<const uint4*>(vb + (int64_t)ja * st_bytes + col);
    const uint4 kb2 = *reinterpret_cast<const uint4*>(kb + (int64_t)jb * st_bytes + col);
    const uint4 vb2 = *reinterpret_cast<const uint4*>(vb + (int64_t)jb * st_bytes + col);
    *reinterpret_cast<uint4*>(k_out + (row0 + i) * ROW_BYTES + col) = ka;
    *reinterpret_cast<uint4*>(v_out + (row0 + i) * ROW_BYTES + col) = va;
    if (i2 < n_keep) {
      *reinterpret_cast<uint4*>(k_out + (row0 + i2) * ROW_BYTES + col) = kb2;
      *reinterpret_cast<uint4*>(v_out + (row0 + i2) * ROW_BYTES + col) = vb2;
    }
  }
}

template <int ROW_BYTES>
static void launch_emit(dim3 grid, hipStream_t st, SelGeom sg, const SeqTab& tab, const float* pooled,
                        const uint4* state, const uint2* slice_cnt, const int64_t* offsets,
                        const void* k, const void* v, const Geom& g, int esize, int32_t* kept_idx,
                        void* k_out, void* v_out, int64_t out_rows, int32_t* status) {
  hipLaunchKernelGGL((sel_emit_kernel<ROW_BYTES>), grid, dim3(256), 0, st, sg, tab, pooled, state,
                     slice_cnt, offsets, (const char*)k, (const char*)v, g.sl * esize, g.sh * esize,
                     g.st * esize, kept_idx, (char*)k_out, (char*)v_out, out_rows, status);
}

int launch_select_compact(const HostCfg& hc, const WsLayout& lay, const float* pooled,
                          const int32_t* budgets, const int64_t* offsets, const void* k,
                          const void* v, int32_t* kept_idx, void* k_out, void* v_out,
                          int64_t out_rows, int32_t* status, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  const SeqTab tab = tiles_for(hc.seq, kSliceElems, 0);
  SelGeom sg{g.n_layers, g.n_kv_heads, g.total_tokens, lay.max_slices};
  unsigned* hist = reinterpret_cast<unsigned*>(ws + lay.hist);
  unsigned* cnt = reinterpret_cast<unsigned*>(ws + lay.sel_cnt);
  uint4* state = reinterpret_cast<uint4*>(ws + lay.sel_state);
  uint2* slice_cnt = reinterpret_cast<uint2*>(ws + lay.slice_cnt);
  dim3 grid(tab.tile0[tab.n_seqs], g.n_kv_heads, g.n_layers);
  stage_mark(kStHist0, st);
  hipLaunchKernelGGL(sel_hist_kernel<0>, grid, dim3(256), 0, st, sg, tab, pooled, budgets, hist, cnt, state, status);
  stage_mark(kStHist1, st);
  hipLaunchKernelGGL(sel_hist_kernel<1>, grid, dim3(256), 0, st, sg, tab, pooled, budgets, hist, cnt, state, status);
  stage_mark(kStHist2, st);
  hipLaunchKernelGGL(sel_hist_kernel<2>, grid, dim3(256), 0, st, sg, tab, pooled, budgets, hist, cnt, state, status);
  stage_mark(kStCount, st);
  hipLaunchKernelGGL(sel_count_kernel, grid, dim3(256), 0, st, sg, tab, pooled, (const uint4*)state, slice_cnt);
  stage_mark(kStEmit, st);
  const int esize = g.f32 ? 4 : 2;
  const int row_bytes = g.head_dim * esize;
  if (row_bytes == 128)
    launch_emit<128>(grid, st, sg, tab, pooled, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else if (row_bytes == 256)
    launch_emit<256>(grid, st, sg, tab, pooled, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else if (row_bytes == 512)
    launch_emit<512>(grid, st, sg, tab, pooled, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else
    return LUKV_EDTYPE;
  return check_launch();
}

}  // namespace lukv
