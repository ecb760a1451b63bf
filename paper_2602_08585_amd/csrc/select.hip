// Steps 3 and 4: per-head top-b_{l,h} by the metric (Sec. 3.2, M^pi(k); Sec. 4.3 "Eviction")
// with the fixed tie rule App. A.1 assumes (lowest position first), and the gather of the
// retained rows into a dense per-head cache (Sec. 3.2, Eq. 3).
//
// Exact radix select on order-preserving 32-bit keys: an 11-bit top digit, then up to two
// digits over the bits in which the surviving keys still differ.
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
#include <string.h>

#include "alloc_device.hpp"
#include "lukv_internal.hpp"

namespace lukv {

__device__ __forceinline__ unsigned key_of(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;  // -0 and +0 tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Histogram increment that does not serialise when a whole wave hits one bin (pooled scores
// come in runs of equal values, and a narrow score range puts every key in the same digit).
__device__ __forceinline__ void hist_add(unsigned* lh, unsigned bin, bool act) {
  const unsigned long long m = __ballot(act);
  if (m == 0ull) return;
  const int leader = __ffsll((long long)m) - 1;
  const unsigned first = (unsigned)__shfl((int)bin, leader);
  if (__ballot(act && bin != first) == 0ull) {
    if ((int)(threadIdx.x & 63) == leader) atomicAdd(&lh[first], (unsigned)__popcll(m));
  } else if (act) {
    atomicAdd(&lh[bin], 1u);
  }
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
__global__ __launch_bounds__(1024) void sel_hist_kernel(SelGeom sg, SeqTab tab, AllocIO aio,
                                                        int n_alloc_blocks, const float* src_scores,
                                                        float* pooled_out, unsigned* hist_parts,
                                                        int32_t* status) {
  __shared__ __align__(16) char scratch[32768];
  unsigned* lh = reinterpret_cast<unsigned*>(scratch);                      // kHistBins counters
  float* rawt = reinterpret_cast<float*>(scratch + kHistBins * 4);           // slice + pool halo
  if ((int)blockIdx.x < n_alloc_blocks) {
    // extra workgroups of the fused path: budgets of one allocation problem each
    if (blockIdx.y == 0 && blockIdx.z == 0) alloc_phase_b(aio, blockIdx.x, scratch, (int)sizeof(scratch));
    return;
  }
  int seq, sl;
  find_tile(tab, blockIdx.x - n_alloc_blocks, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z, t = threadIdx.x;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const int64_t base = ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const float* src = src_scores + base;
  float* pooled = POOL ? pooled_out + base : nullptr;
  unsigned* my_part = hist_parts + ((int64_t)hi * sg.max_slices + sl) * (kHistBins / 2);
  // the selection status word starts at zero; later kernels of the call only OR into it
  if (t == 0 && (int)blockIdx.x == n_alloc_blocks && blockIdx.y == 0 && blockIdx.z == 0) *status = 0;

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
  hist_add(lh, key_of(s) >> 21, j < L);
  __syncthreads();
  my_part[t] = (lh[2 * t] & 0xFFFFu) | (lh[2 * t + 1] << 16);   // counts <= 1024 fit 16 bits
}

// One workgroup per head: fixes the threshold key T and the number of ties to keep,
// state[hi] = {T, ties at T to keep, budget after clamping, 0}, counts per block of 256
// scores, and (if offsets_out is given) this head's row offset = sum of the budgets before it.
// A thread owns the keys j = r*32768 + u*1024 + t (u < 32) of round r; with ONE (L <= 32768)
// they are loaded once, all 32 loads in flight together, and stay in registers for every
// phase; longer heads re-read them round by round.
template <bool ONE>
__global__ __launch_bounds__(1024) void sel_tail_kernel(SelGeom sg, SeqTab tab, const float* scores,
                                                        const int32_t* budgets, const unsigned* hist_parts,
                                                        uint4* state, uint2* block_cnt,
                                                        int64_t* offsets_out, int n_heads_total,
                                                        int32_t* status) {
  constexpr int KPT = 32;
  __shared__ unsigned lh[kHistBins];
  __shared__ unsigned part[16];
  __shared__ unsigned sel[2];
  __shared__ long long osum[16];
  __shared__ unsigned short cg[16][KPT], ce[16][KPT];
  const int hi = blockIdx.x, t = threadIdx.x;
  const int kvh = hi % sg.n_kv_heads, layer = (hi / sg.n_kv_heads) % sg.n_layers;
  const int seq = hi / (sg.n_kv_heads * sg.n_layers);
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int n_slices = (L + kSliceElems - 1) / kSliceElems;
  const int n_rounds = (L + 1024 * KPT - 1) / (1024 * KPT);
  const float* keys_src = scores + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const int lane = t & 63, wave = t >> 6;

  unsigned key[KPT];   // order-preserving keys of this thread's scores (0 beyond L: below every real key's use)
  auto load_round = [&](int r) {
    float f[KPT];
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const int jj = (r * KPT + u) * 1024 + t;
      f[u] = jj < L ? keys_src[jj] : 0.f;
    }
#pragma unroll
    for (int u = 0; u < KPT; ++u) key[u] = key_of(f[u]);
  };
  if (ONE) load_round(0);

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
    for (int s0 = 0; s0 < n_slices; s0 += 32) {
      unsigned w[32];   // independent loads first: one memory latency per 32 slices
#pragma unroll
      for (int u = 0; u < 32; ++u) w[u] = s0 + u < n_slices ? hp[(int64_t)(s0 + u) * (kHistBins / 2)] : 0u;
#pragma unroll
      for (int u = 0; u < 32; ++u) { c_lo += w[u] & 0xFFFFu; c_hi += w[u] >> 16; }
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
  // The keys that share digit 0 usually differ only in some low bits: find the bits in which
  // they vary at all and spread those over the remaining digits (at most 11 + 10 bits), so
  // that a narrow range of scores still fills the histogram evenly.
  if (t < 2) sel[t] = t == 0 ? 0xFFFFFFFFu : 0u;   // min, max of the candidate keys
  __syncthreads();
  {
    unsigned cmin = 0xFFFFFFFFu, cmax = 0u;
    for (int r = 0; r < n_rounds; ++r) {
      if (!ONE) load_round(r);
#pragma unroll
      for (int u = 0; u < KPT; ++u)
        if ((r * KPT + u) * 1024 + t < L && (key[u] >> 21) == (prefix >> 21)) {
          cmin = key[u] < cmin ? key[u] : cmin;
          cmax = key[u] > cmax ? key[u] : cmax;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const unsigned a2 = (unsigned)__shfl_xor((int)cmin, o), b2 = (unsigned)__shfl_xor((int)cmax, o);
      cmin = a2 < cmin ? a2 : cmin;
      cmax = b2 > cmax ? b2 : cmax;
    }
    if (lane == 0) { atomicMin(&sel[0], cmin); atomicMax(&sel[1], cmax); }
  }
  __syncthreads();
  const unsigned cand_min = sel[0], vary = sel[0] ^ sel[1];
  __syncthreads();
  if (vary == 0u) {
    prefix = cand_min;             // every candidate is the same key: T is that key, `want` ties
  } else {
    const int vb = 31 - __clz(vary);                    // top varying bit (<= 20)
    const int shift1 = vb > 10 ? vb - 10 : 0;           // digit 1: bits vb .. shift1
    const unsigned mask1 = (2u << (vb - shift1)) - 1u;
    prefix = cand_min & ~((2u << vb) - 1u);             // bits above vb are common
    lh[t] = 0;
    lh[t + 1024] = 0;
    __syncthreads();
    for (int r = 0; r < n_rounds; ++r) {
      if (!ONE) load_round(r);
#pragma unroll
      for (int u = 0; u < KPT; ++u)
        if ((r * KPT + u) * 1024 + t < L && (key[u] >> (vb + 1)) == (prefix >> (vb + 1)))
          atomicAdd(&lh[(key[u] >> shift1) & mask1], 1u);
    }
    __syncthreads();
    {
      const unsigned a1 = lh[2047 - 2 * t], a0 = lh[2046 - 2 * t];
      const unsigned before = scan1024(a1 + a0, part);
      if (before < want && want <= before + a1) { sel[0] = 2047 - 2 * t; sel[1] = want - before; }
      else if (before + a1 < want && want <= before + a1 + a0) { sel[0] = 2046 - 2 * t; sel[1] = want - before - a1; }
      __syncthreads();
      prefix |= sel[0] << shift1;
      want = sel[1];
    }
    if (shift1 > 0) {
      // digit 2: the remaining low bits (at most 10)
      __syncthreads();
      lh[t] = 0;
      __syncthreads();
      const unsigned mask2 = (1u << shift1) - 1u;
      for (int r = 0; r < n_rounds; ++r) {
        if (!ONE) load_round(r);
#pragma unroll
        for (int u = 0; u < KPT; ++u)
          if ((r * KPT + u) * 1024 + t < L && (key[u] >> shift1) == (prefix >> shift1))
            atomicAdd(&lh[key[u] & mask2], 1u);
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
    }
  }
  const unsigned T = prefix;
  if (t == 0) state[hi] = make_uint4(T, want, (unsigned)kb, 0u);
  // per block of 256 scores: keys above T and keys equal to T.  Key (r, u, t) sits in block
  // (r*KPT + u)*4 + t/256: four waves share a block, ballots count, LDS joins the four.
  for (int r = 0; r < n_rounds; ++r) {
    if (!ONE) load_round(r);
    __syncthreads();
#pragma unroll
    for (int u = 0; u < KPT; ++u) {
      const bool in = (r * KPT + u) * 1024 + t < L;
      const unsigned long long mg = __ballot(in && key[u] > T), me = __ballot(in && key[u] == T);
      if (lane == 0) { cg[wave][u] = (unsigned short)__popcll(mg); ce[wave][u] = (unsigned short)__popcll(me); }
    }
    __syncthreads();
    if (t < 4 * KPT) {
      const int u = t >> 2, q = t & 3;
      const int b = (r * KPT + u) * 4 + q;
      if (b * kEmitElems < L) {
        unsigned gt = 0, eq = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) { gt += cg[4 * q + w][u]; eq += ce[4 * q + w][u]; }
        block_cnt[(int64_t)hi * sg.max_blocks + b] = make_uint2(gt, eq);
      }
    }
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
int launch_select_compact(const HostCfg& hc, const WsLayout& lay, const AllocIO* aio,
                          const float* scores_in, bool pool,
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
  AllocIO io;
  memset(&io, 0, sizeof(io));
  int n_alloc = 0;
  if (aio) { io = *aio; n_alloc = aio->n_problems; }
  dim3 gridH(tabH.tile0[tabH.n_seqs] + n_alloc, g.n_kv_heads, g.n_layers);
  dim3 gridE(tabE.tile0[tabE.n_seqs], g.n_kv_heads, g.n_layers);
  stage_mark(kStHist, st);
  if (pool)
    hipLaunchKernelGGL(sel_hist_kernel<true>, gridH, dim3(1024), 0, st, sg, tabH, io, n_alloc, scores_in,
                       pooled_out, hist, status);
  else
    hipLaunchKernelGGL(sel_hist_kernel<false>, gridH, dim3(1024), 0, st, sg, tabH, io, n_alloc, scores_in,
                       (float*)nullptr, hist, status);
  const float* sel_scores = pool ? pooled_out : scores_in;
  stage_mark(kStTail, st);
  if (hc.max_len <= 32768)
    hipLaunchKernelGGL(sel_tail_kernel<true>, dim3(hc.n_hi), dim3(1024), 0, st, sg, tabH, sel_scores, budgets,
                       (const unsigned*)hist, state, block_cnt, make_offsets ? offsets : (int64_t*)nullptr,
                       hc.n_hi, status);
  else
    hipLaunchKernelGGL(sel_tail_kernel<false>, dim3(hc.n_hi), dim3(1024), 0, st, sg, tabH, sel_scores, budgets,
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
