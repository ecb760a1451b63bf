// Steps 3 and 4: per-head top-b_{l,h} by the metric (Sec. 3.2, M^pi(k); Sec. 4.3 "Eviction")
// with the fixed tie rule App. A.1 assumes (lowest position first), and the gather of the
// retained rows into a dense per-head cache (Sec. 3.2, Eq. 3).
//
// Exact radix select on order-preserving 32-bit keys.  The first digit is scaled to the range
// of the head's metric: bin(key) = min((key - lo) >> shift, 2047), any non-decreasing map of
// the key serves, so that the bin holding the k-th largest key holds few keys (the threshold
// candidates) whatever the spread of the scores.
//   sel_range - stand-alone scores only: (min, max) of the finite scores per slice (the fused
//               path gets the range of the metric from the score kernel that produced it).
//   sel_hist  - one workgroup (1024 threads) per slice of 1024 scores: [optionally the clipped
//               max-pool + forced +inf of step 1,] an LDS histogram of the first digit, stored
//               as the slice's own 16-bit suffix counts S[b] = #(keys of the slice in bins >= b)
//               (no shared hot counters).
//   sel_tail  - one workgroup per head: sums the suffix counts over the slices (which gives
//               the bin T0 of the k-th key without a scan, and by one look-up per slice the
//               rows above that bin), collects the candidates of bin T0, resolves the exact
//               threshold key T among them with up to two further adaptive digits, and
//               leaves, per slice, the kept rows and the ties before it.
//   sel_emit  - one workgroup per slice: keep (key > T) plus the first r ties by position,
//               write ascending positions and copy the K and V rows (16 bytes per lane).
// Calls with many heads and sequences of at most 32768 tokens take the whole-head form instead
// (sel_head, sel_gather, further below): one workgroup per head keeps the head's keys in
// registers and leaves a keep mask, a gather kernel copies the rows.
// No counter, flag or fence between workgroups anywhere: kernel boundaries order the phases.
#include <string.h>

#include "alloc_device.hpp"
#include "lukv_internal.hpp"

namespace lukv {

constexpr int kCandLds = 4096;   // threshold candidates a head keeps in LDS (more: workspace)

__device__ __forceinline__ unsigned key_of(float f) {
  unsigned u = __float_as_uint(f);
  if (u == 0x80000000u) u = 0u;  // -0 and +0 tie
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// first digit: non-decreasing in the key, clamped at both ends
__device__ __forceinline__ unsigned bin_of(unsigned key, unsigned lo, unsigned shift) {
  const unsigned d = key > lo ? (key - lo) >> shift : 0u;
  return d < (unsigned)(kHistBins - 1) ? d : (unsigned)(kHistBins - 1);
}

// Histogram increment that returns the key's rank inside its bin (arrival order) and does not
// serialise when a whole wave hits one bin (pooled scores come in runs of equal values).
__device__ __forceinline__ unsigned hist_add(unsigned* lh, unsigned bin, bool act) {
  const unsigned long long m = __ballot(act);
  if (m == 0ull) return 0u;
  const int lane = threadIdx.x & 63;
  const int leader = __ffsll((long long)m) - 1;
  const unsigned first = (unsigned)__shfl((int)bin, leader);
  if (__ballot(act && bin != first) == 0ull) {
    unsigned at = 0;
    if (lane == leader) at = atomicAdd(&lh[first], (unsigned)__popcll(m));
    return (unsigned)__shfl((int)at, leader) + (unsigned)__popcll(m & ((1ull << lane) - 1ull));
  }
  return act ? atomicAdd(&lh[bin], 1u) : 0u;
}

struct SelGeom {
  int32_t n_layers, n_kv_heads, total_tokens, max_slices;
  int32_t window, pool_kernel, n_sink;
  int32_t range_chunk;    // positions covered by one group of range entries
  int32_t range_per;      // entries per group
  int32_t range_tail;     // trailing positions without entries (the window, fused path)
  int32_t range_stride;   // entries per head in the range array
  int32_t slices_per_wg;  // slices one workgroup of sel_hist takes
};

// (min, max) of the finite scores of every slice, for scores that come from the caller.
__global__ __launch_bounds__(1024) void sel_range_kernel(SelGeom sg, SeqTab tab, const float* scores,
                                                         float2* range) {
  __shared__ float mn_s[16], mx_s[16];
  int seq, sl;
  find_tile(tab, blockIdx.x, seq, sl);
  const int kvh = blockIdx.y, layer = blockIdx.z, t = threadIdx.x;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const float* src = scores + ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const int j = sl * kSliceElems + t;
  const float s = j < L ? src[j] : INFINITY;
  const bool fin = j < L && fabsf(s) < INFINITY;     // false for NaN too
  float mn = fin ? s : INFINITY, mx = fin ? s : -INFINITY;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    mn = fminf(mn, __shfl_xor(mn, o));
    mx = fmaxf(mx, __shfl_xor(mx, o));
  }
  if ((t & 63) == 0) { mn_s[t >> 6] = mn; mx_s[t >> 6] = mx; }
  __syncthreads();
  if (t == 0) {
    for (int w = 1; w < 16; ++w) { mn = fminf(mn, mn_s[w]); mx = fmaxf(mx, mx_s[w]); }
    range[(int64_t)hi * sg.range_stride + sl] = make_float2(mn, mx);
  }
}

// Slice histogram of the first digit (and, with POOL, the pooled scores themselves).
template <bool POOL>
__global__ __launch_bounds__(1024) void sel_hist_kernel(SelGeom sg, SeqTab tab, AllocIO aio,
                                                        int n_alloc_blocks, const float* src_scores,
                                                        float* pooled_out, const float2* range,
                                                        unsigned* hist_parts, uint2* head_dig,
                                                        unsigned long long* by_bin, int32_t* status) {
  __shared__ __align__(16) char scratch[kAllocLdsBytes];
  unsigned* lh = reinterpret_cast<unsigned*>(scratch);                      // kHistBins counters
  float* rawt = reinterpret_cast<float*>(scratch + kHistBins * 4);           // slice + pool halo
  unsigned* part = reinterpret_cast<unsigned*>(scratch + kHistBins * 4 + 4352);
  unsigned* rng = part + 16;                                                 // min key, max key
  if ((int)blockIdx.x < n_alloc_blocks) {
    // extra workgroups of the fused path: budgets of one allocation problem each
    if (blockIdx.y == 0 && blockIdx.z == 0) alloc_phase_b(aio, blockIdx.x, scratch, (int)sizeof(scratch));
    return;
  }
  int seq, tile;
  find_tile(tab, blockIdx.x - n_alloc_blocks, seq, tile);
  const int kvh = blockIdx.y, layer = blockIdx.z, t = threadIdx.x;
  const int lane = t & 63;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  const int64_t base = ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const float* src = src_scores + base;
  float* pooled = POOL ? pooled_out + base : nullptr;
  // the selection status word starts at zero; later kernels of the call only OR into it
  if (t == 0 && (int)blockIdx.x == n_alloc_blocks && blockIdx.y == 0 && blockIdx.z == 0) *status = 0;

  if (t < 2) rng[t] = t == 0 ? 0xFFFFFFFFu : 0u;
  const int P = L - sg.window, h = sg.pool_kernel >> 1;
  const int n_slices = (L + kSliceElems - 1) / kSliceElems;
  // a workgroup takes sg.slices_per_wg consecutive slices (more than one in calls with
  // thousands of slices: fewer, longer workgroups)
  // this thread's inputs of a slice: with POOL the raw metric at j0 - h + t and (for the halo)
  // at j0 - h + 1024 + t, otherwise its own score; fetched one slice ahead, the first one before
  // anything else so that it is in flight while the head's range is folded
  const int sl_end = min(n_slices, (tile + 1) * sg.slices_per_wg);
  auto fetch = [&](int sl, float& a, float& b) {
    const int j0 = sl * kSliceElems;
    if (POOL) {
      const int ja = j0 - h + t, jb = ja + 1024;
      a = (ja >= 0 && ja < P) ? src[ja] : -INFINITY;
      b = (t < 2 * h && jb < P) ? src[jb] : -INFINITY;
    } else {
      a = j0 + t < L ? src[j0 + t] : 0.f;
      b = 0.f;
    }
  };
  float in_a, in_b;
  fetch(tile * sg.slices_per_wg, in_a, in_b);
  // range of the head's metric: every workgroup of the head folds the same entries
  float mn = INFINITY, mx = -INFINITY;
  {
    const int n_ent = (L - sg.range_tail + sg.range_chunk - 1) / sg.range_chunk * sg.range_per;
    const float2* rp = range + (int64_t)hi * sg.range_stride;
    if ((t & ~63) < n_ent) {
      for (int e = t; e < n_ent; e += 1024) {
        const float2 r = rp[e];
        mn = fminf(mn, r.x);
        mx = fmaxf(mx, r.y);
      }
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        mn = fminf(mn, __shfl_xor(mn, o));
        mx = fmaxf(mx, __shfl_xor(mx, o));
      }
    }
  }
  __syncthreads();
  if (lane == 0 && mn <= mx) { atomicMin(&rng[0], key_of(mn)); atomicMax(&rng[1], key_of(mx)); }
  __syncthreads();
  unsigned lo = 0u, shift = 21u;   // without a usable range: the top 11 bits of the key
  if (rng[0] <= rng[1]) {
    const unsigned span = rng[1] - rng[0];
    const int bits = span ? 32 - __clz(span) : 0;
    lo = rng[0];
    shift = bits > 11 ? (unsigned)(bits - 11) : 0u;
  }
  if (t == 0 && tile == 0) head_dig[hi] = make_uint2(lo, shift);   // the head's first digit, for sel_tail
  for (int sl = tile * sg.slices_per_wg; sl < sl_end; ++sl) {
    unsigned* my_part = hist_parts + ((int64_t)hi * sg.max_slices + sl) * (kHistBins / 2);
    const int j0 = sl * kSliceElems, j = j0 + t;
    lh[t] = 0;
    lh[t + 1024] = 0;
    float s = in_a;
    if (POOL) {
      rawt[t] = in_a;
      if (t < 2 * h) rawt[1024 + t] = in_b;
    }
    if (sl + 1 < sl_end) fetch(sl + 1, in_a, in_b);   // in flight during this slice's work
    __syncthreads();   // counters cleared, halo staged
    if (POOL && j < L) {
      // clipped max-pool over the prefix [0, P); window and sink positions are forced to +inf
      s = INFINITY;
      if (j >= sg.n_sink && j < P) {
        s = rawt[t];
        for (int d = 1; d <= 2 * h; ++d) s = fmaxf(s, rawt[t + d]);
      }
      pooled[j] = s;
    }
    const unsigned key = key_of(s), bin = bin_of(key, lo, shift);
    const unsigned rank = hist_add(lh, bin, j < L);
    __syncthreads();
    // suffix counts, descending bins: thread t owns bins 2047-2t and 2046-2t (packed word 1023-t)
    const unsigned a1 = lh[2047 - 2 * t], a0 = lh[2046 - 2 * t];
    const unsigned above = block_scan_u32(a1 + a0, part);
    const unsigned s_hi = above + a1, s_lo = s_hi + a0;          // <= 1024: fit 16 bits
    my_part[1023 - t] = s_lo | (s_hi << 16);
    // the slice's (key, position) pairs ordered by descending bin: the keys of bin b sit at
    // [S[b+1], S[b]), so whoever knows the threshold bin reads its candidates directly
    __syncthreads();
    lh[2047 - 2 * t] = above;
    lh[2046 - 2 * t] = s_hi;
    __syncthreads();
    if (j < L) by_bin[base + j0 + lh[bin] + rank] = ((unsigned long long)key << 32) | (unsigned)j;
    __syncthreads();   // lh and the halo are rewritten by the next slice
  }
}

// Exact threshold T among the n_c candidates of the list (the want-th largest, ties included)
// by digits over the open bits of the bin's key interval, and per-slice counts of candidates
// above and at T.  Entries are (key << 32) | position.  All threads call it.
template <class List>
__device__ __forceinline__ void tail_resolve(List list, unsigned n_c, unsigned want, bool interior,
                                             unsigned bin_base, unsigned bin_bits, unsigned* lh,
                                             unsigned* part, unsigned* sel, unsigned* s_gt,
                                             unsigned* s_eq, unsigned& T_out, unsigned& r_eq_out) {
  const int t = threadIdx.x, lane = t & 63;
  // The candidates lie in [base, base + 2^rest).  An interior bin is such an interval by
  // construction; a clamped end bin is not, and its candidates' minimum and maximum are taken.
  unsigned base = bin_base;
  int rest = (int)bin_bits;
  if (!interior) {
    unsigned cmin = 0xFFFFFFFFu, cmax = 0u;
    for (unsigned i = t; i < n_c; i += 1024) {
      const unsigned key = (unsigned)(list[i] >> 32);
      cmin = key < cmin ? key : cmin;
      cmax = key > cmax ? key : cmax;
    }
    if ((unsigned)(t & ~63) < n_c) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const unsigned a2 = (unsigned)__shfl_xor((int)cmin, o), b2 = (unsigned)__shfl_xor((int)cmax, o);
        cmin = a2 < cmin ? a2 : cmin;
        cmax = b2 > cmax ? b2 : cmax;
      }
      if (lane == 0) { atomicMin(&sel[0], cmin); atomicMax(&sel[1], cmax); }
    }
    __syncthreads();
    base = sel[0];
    const unsigned span = sel[1] - sel[0];
    rest = span ? 32 - __clz(span) : 0;
  }
  // digits of at most 11 bits of (key - base), from the top open bit down
  unsigned prefix = 0u;
  while (rest > 0) {
    const int sh = rest > 11 ? rest - 11 : 0;
    const unsigned mask = (1u << (rest - sh)) - 1u;
    const unsigned hi_mask = rest == 32 ? 0u : ~((1u << rest) - 1u);
    __syncthreads();
    lh[t] = 0;
    lh[t + 1024] = 0;
    __syncthreads();
    for (unsigned i = t; i < n_c; i += 1024) {
      const unsigned dk = (unsigned)(list[i] >> 32) - base;
      if ((dk & hi_mask) == (prefix & hi_mask)) atomicAdd(&lh[(dk >> sh) & mask], 1u);
    }
    __syncthreads();
    const unsigned a1 = lh[2047 - 2 * t], a0 = lh[2046 - 2 * t];
    const unsigned before = block_scan_u32(a1 + a0, part);
    if (before < want && want <= before + a1) { sel[2] = 2047 - 2 * t; sel[3] = want - before; }
    else if (before + a1 < want && want <= before + a1 + a0) { sel[2] = 2046 - 2 * t; sel[3] = want - before - a1; }
    __syncthreads();
    prefix |= sel[2] << sh;
    want = sel[3];
    rest = sh;
  }
  const unsigned T = base + prefix;
  for (unsigned i = t; i < n_c; i += 1024) {
    const unsigned long long e = list[i];
    const unsigned key = (unsigned)(e >> 32), sl = ((unsigned)e) >> 10;
    if (key > T) atomicAdd(&s_gt[sl], 1u);
    else if (key == T) atomicAdd(&s_eq[sl], 1u);
  }
  T_out = T;
  r_eq_out = want;
}

// Candidates of bin T0: slice s holds them at by_bin[s*1024 + start[s] ..] (cnt[s] of them);
// they are copied to list[off[s] ..], two slices per wave at a time.
template <class List>
__device__ __forceinline__ void tail_collect(List list, const unsigned long long* by_bin, int n_slices,
                                             const unsigned* start, const unsigned* cnt,
                                             const unsigned* off) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int s0 = wave; s0 < n_slices; s0 += 16) {
    const unsigned n = cnt[s0], at = off[s0];
    const unsigned long long* src = by_bin + (int64_t)s0 * kSliceElems + start[s0];
    for (unsigned c = lane; c < n; c += 64) list[at + c] = src[c];
  }
}

// One workgroup per head: fixes the threshold key T and the number of ties to keep,
// state[hi] = {T, ties at T to keep, budget after clamping, 0}; per slice the kept rows and
// the ties in earlier slices; and (if offsets_out is given) this head's row offset = sum of
// the budgets before it.
__global__ __launch_bounds__(1024) void sel_tail_kernel(SelGeom sg, SeqTab tab, const int32_t* budgets,
                                                        const unsigned* hist_parts,
                                                        const unsigned long long* by_bin,
                                                        const uint2* head_dig, uint4* state,
                                                        uint2* slice_cnt, unsigned long long* cand_glob,
                                                        int64_t* offsets_out, int n_heads_total,
                                                        int32_t* status) {
  __shared__ unsigned lh[kHistBins];
  __shared__ unsigned part[16];
  __shared__ unsigned sel[4];
  __shared__ unsigned pick[3];
  __shared__ long long osum[16];
  __shared__ unsigned clo[1024], s_gt[1024], s_eq[1024], c_cnt[1024];
  __shared__ unsigned long long cand_lds[kCandLds];
  const int hi = blockIdx.x, t = threadIdx.x;
  const int kvh = hi % sg.n_kv_heads, layer = (hi / sg.n_kv_heads) % sg.n_layers;
  const int seq = hi / (sg.n_kv_heads * sg.n_layers);
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  const int n_slices = (L + kSliceElems - 1) / kSliceElems;     // <= 1024 (checked on the host)
  const int64_t head_base = ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const int lane = t & 63, wave = t >> 6;
  uint2* my_cnt = slice_cnt + (int64_t)hi * sg.max_slices;
  const unsigned* hp = hist_parts + (int64_t)hi * sg.max_slices * (kHistBins / 2) + (1023 - t);

  // loads in flight together: suffix counts of the first 32 slices, budgets
  unsigned w[32];
#pragma unroll
  for (int u = 0; u < 32; ++u) w[u] = u < n_slices ? hp[(int64_t)u * (kHistBins / 2)] : 0u;
  int kb = budgets[hi];
  const uint2 dig = head_dig[hi];
  long long acc = 0;
  // row offsets are sums of the budgets as the selection uses them (clamped to [0, L]), so a
  // budget that the allocation left out of range can never move a later head's rows out of bounds
  const int heads_per_seq = sg.n_kv_heads * sg.n_layers;
  if (offsets_out)
    for (int h2 = t; h2 < hi; h2 += 1024) {
      const int s2 = h2 / heads_per_seq, L2 = tab.cu[s2 + 1] - tab.cu[s2], b2 = budgets[h2];
      acc += b2 < 0 ? 0 : (b2 > L2 ? L2 : b2);
    }

  // suffix counts of the head: thread t owns packed word 1023-t, bins 2047-2t (high half) and
  // 2046-2t; C[b] = keys of the head in bins >= b
  unsigned c_hi = 0, c_lo = 0;
#pragma unroll
  for (int u = 0; u < 32; ++u) { c_lo += w[u] & 0xFFFFu; c_hi += w[u] >> 16; }
  for (int s0 = 32; s0 < n_slices; s0 += 32) {
#pragma unroll
    for (int u = 0; u < 32; ++u) w[u] = s0 + u < n_slices ? hp[(int64_t)(s0 + u) * (kHistBins / 2)] : 0u;
#pragma unroll
    for (int u = 0; u < 32; ++u) { c_lo += w[u] & 0xFFFFu; c_hi += w[u] >> 16; }
  }
  if (offsets_out) {
    if (wave * 64 < hi) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) {
        const int lo2 = __shfl_xor((int)(acc & 0xFFFFFFFFll), o), hi32 = __shfl_xor((int)(acc >> 32), o);
        acc += ((long long)hi32 << 32) | (unsigned)lo2;
      }
    }
    if (lane == 0) osum[wave] = acc;
  }
  clo[t] = c_lo;
  if (t < 2) sel[t] = t == 0 ? 0xFFFFFFFFu : 0u;   // min, max of the candidate keys
  __syncthreads();
  if (offsets_out && t == 0) {
    long long tot = 0;
    for (int w2 = 0; w2 < 16; ++w2) tot += osum[w2];
    offsets_out[hi] = tot;
    if (hi == n_heads_total - 1) offsets_out[n_heads_total] = tot + (kb < 0 ? 0 : (kb > L ? L : kb));
  }
  if (kb < 0 || kb > L) {
    if (t == 0) atomicOr(status, LUKV_ST_CLAMPED);
    kb = kb < 0 ? 0 : L;
  }
  // a head that keeps nothing runs the same code with k = 1 and overrides the result
  const bool keep_none = kb == 0;
  if (keep_none) kb = 1;
  // T0 = the largest bin with C[T0] >= kb; C is non-increasing in the bin, so exactly one
  // thread sees the step.  `want` keys are still needed from bin T0.
  {
    const unsigned above = t ? clo[t - 1] : 0u;    // C[2048 - 2t]
    const unsigned k = (unsigned)kb;
    if (c_hi >= k && above < k) { pick[0] = 2047 - 2 * t; pick[1] = k - above; pick[2] = c_hi - above; }
    else if (c_lo >= k && c_hi < k) { pick[0] = 2046 - 2 * t; pick[1] = k - c_hi; pick[2] = c_lo - c_hi; }
  }
  __syncthreads();
  const unsigned T0 = pick[0], want0 = pick[1], n_cand = pick[2];
  // per slice, from its suffix counts: rows above bin T0, and where its candidates sit
  unsigned n_s = 0;
  if (t < n_slices) {
    const unsigned* sp = hist_parts + ((int64_t)hi * sg.max_slices + t) * (kHistBins / 2);
    const unsigned w0 = sp[T0 >> 1];
    unsigned up, dn;   // S[T0 + 1], S[T0]
    if (T0 & 1u) {
      dn = w0 >> 16;
      up = T0 == (unsigned)(kHistBins - 1) ? 0u : (sp[(T0 >> 1) + 1] & 0xFFFFu);
    } else {
      dn = w0 & 0xFFFFu;
      up = w0 >> 16;
    }
    n_s = dn - up;
    s_gt[t] = up;
    s_eq[t] = 0u;
    c_cnt[t] = n_s;
  }
  unsigned* c_off = clo;   // free after the pick above
  if (n_slices <= 64) {
    if (wave == 0) c_off[lane] = wave_scan_incl(n_s) - n_s;
  } else {
    const unsigned o = block_scan_u32(n_s, part);
    c_off[t] = o;
  }
  __syncthreads();
  // key interval of bin T0 (the two end bins are clamped and have none)
  const bool interior = T0 > 0u && T0 < (unsigned)(kHistBins - 1);
  const unsigned bin_base = dig.x + (T0 << dig.y);
  unsigned T, r_eq;
  if (n_cand <= (unsigned)kCandLds) {
    tail_collect(cand_lds, by_bin + head_base, n_slices, s_gt, c_cnt, c_off);
    __syncthreads();
    tail_resolve(cand_lds, n_cand, want0, interior, bin_base, dig.y, lh, part, sel, s_gt, s_eq, T, r_eq);
  } else {
    unsigned long long* list = cand_glob + head_base;
    tail_collect(list, by_bin + head_base, n_slices, s_gt, c_cnt, c_off);
    __syncthreads();
    tail_resolve(list, n_cand, want0, interior, bin_base, dig.y, lh, part, sel, s_gt, s_eq, T, r_eq);
  }
  __syncthreads();
  // nothing kept: a threshold above every key and no ties
  if (t == 0) state[hi] = keep_none ? make_uint4(0xFFFFFFFFu, 0u, 0u, 0u) : make_uint4(T, r_eq, (unsigned)kb, 0u);
  if (n_slices <= 64) {
    if (wave == 0) {
      const unsigned g = lane < n_slices && !keep_none ? s_gt[lane] : 0u;
      const unsigned e = lane < n_slices && !keep_none ? s_eq[lane] : 0u;
      const unsigned g_before = wave_scan_incl(g) - g, e_before = wave_scan_incl(e) - e;
      if (lane < n_slices) my_cnt[lane] = make_uint2(g_before, e_before);
    }
  } else {
    const unsigned g = t < n_slices && !keep_none ? s_gt[t] : 0u;
    const unsigned e = t < n_slices && !keep_none ? s_eq[t] : 0u;
    const unsigned g_before = block_scan_u32(g, part);
    const unsigned e_before = block_scan_u32(e, part);
    if (t < n_slices) my_cnt[t] = make_uint2(g_before, e_before);
  }
}

constexpr int kEmitElems = 256;    // scores one workgroup of the emit/gather kernel owns

// One workgroup per block of 256 scores, four blocks to a slice.  The rows kept before the
// slice come from sel_tail; the (up to three) earlier blocks of the slice are re-judged here.
template <int ROW_BYTES>
__global__ __launch_bounds__(256) void sel_emit_kernel(SelGeom sg, SeqTab tab, const float* scores,
                                                       const uint4* state, const uint2* slice_cnt,
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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int sl = blk >> 2, q = blk & 3;
  const int j = blk * kEmitElems + threadIdx.x;
  const bool in = j < L;
  // scores of this block and of the earlier blocks of the slice (those are full blocks)
  float fq[3];
#pragma unroll
  for (int p = 0; p < 3; ++p) fq[p] = p < q ? src[sl * kSliceElems + p * kEmitElems + (int)threadIdx.x] : 0.f;
  const unsigned key = in ? key_of(src[j]) : 0u;
  const uint4 stt = state[hi];
  const uint2 before = slice_cnt[(int64_t)hi * sg.max_slices + sl];
  const int64_t head_row0 = offsets[hi];
  const unsigned T = stt.x, r_eq = stt.y;

  unsigned pg = 0, pe = 0;
#pragma unroll
  for (int p = 0; p < 3; ++p) {
    const unsigned kp = key_of(fq[p]);
    pg += (unsigned)__popcll(__ballot(p < q && kp > T));
    pe += (unsigned)__popcll(__ballot(p < q && kp == T));
  }
  const bool is_eq = in && key == T;
  const unsigned long long em = __ballot(is_eq);
  if (lane == 0) { red_g[wave] = pg; red_e[wave] = pe; weq[wave] = (unsigned)__popcll(em); }
  __syncthreads();
  const unsigned gt_before = before.x + red_g[0] + red_g[1] + red_g[2] + red_g[3];
  const unsigned eq_before = before.y + red_e[0] + red_e[1] + red_e[2] + red_e[3];
  const int64_t row0 = head_row0 + gt_before + (eq_before < r_eq ? eq_before : r_eq);

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
  // a head whose row offset is negative (caller-supplied offsets) writes nothing at all
  const bool before_start = head_row0 < 0;
  if (keep) {
    list[pos] = j;
    if (!before_start && row0 + pos < out_rows) kept_idx[row0 + pos] = j;
  }
  __syncthreads();

  // rows outside [0, out_rows) are dropped and flagged, never written
  if (before_start || row0 + n_keep > out_rows) {
    if (threadIdx.x == 0) atomicOr(status, LUKV_ST_CLAMPED);
    n_keep = before_start ? 0u : (row0 < out_rows ? (unsigned)(out_rows - row0) : 0u);
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

// ---- whole-head selection for sequences of up to kSelHeadMaxLen tokens -------------------
//
// One workgroup of 1024 threads owns a head: thread t owns the run of positions [32t, 32t + 32).
// The head's scores pass through LDS once (coalesced loads, one padded row per run, so that a
// thread reads its run and the pooling halo without bank conflicts); pooled scores and keys then
// live in registers, and every later step (range of the metric, first digit, further digits
// among the keys of the threshold bin, tie ranks by position, row prefixes) is a pass over those
// 32 registers plus a workgroup scan.  The result is one 32-bit keep mask per run and the number
// of kept rows before the run: the gather kernel needs nothing else.
constexpr int kHeadRun = 32;                          // positions per thread
constexpr int kSelHeadMaxLen = 1024 * kHeadRun;       // longest sequence this form takes
constexpr int kHeadRunLds = kHeadRun + 1;             // LDS words per run (odd stride)
constexpr int kHeadPrefixStride = 1024 + 8;           // runpre entries per head (entry 1024 = total)
constexpr int kHeadStageWords = 1026 * kHeadRunLds;   // runs -1 .. 1024 (the two outer ones hold -inf)
constexpr int kSelHeadLdsBytes = kHeadStageWords * 4 + kHistBins * 4 + 512;

__device__ __forceinline__ unsigned umin_op(unsigned a, unsigned b) { return a < b ? a : b; }
__device__ __forceinline__ unsigned umax_op(unsigned a, unsigned b) { return a > b ? a : b; }

// Reduction of one unsigned per thread over a workgroup of 16 waves; every thread gets the
// result.  red has 16 slots; two barriers inside.
template <class Op>
__device__ __forceinline__ unsigned block_reduce_u32(unsigned v, unsigned ident, Op op, unsigned* red) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  v = wave_reduce_to_last(v, ident, op);
  __syncthreads();
  if (lane == 63) red[wave] = v;
  __syncthreads();
  unsigned r = lane < 16 ? red[lane] : ident;
  r = wave_reduce_to_last(r, ident, op);
  return (unsigned)__builtin_amdgcn_readlane((int)r, 63);
}

// first digit of a key known to be a real key or 0: (key - lo, saturating) >> shift, clamped
__device__ __forceinline__ unsigned head_bin(unsigned key, unsigned lo, unsigned shift) {
  const unsigned d = (key > lo ? key - lo : 0u) >> shift;
  return d < (unsigned)(kHistBins - 1) ? d : (unsigned)(kHistBins - 1);
}

// Suffix scan of the histogram (descending bins) and the bin that holds the want-th largest
// key: pick[0] = bin, pick[1] = keys still wanted from that bin.
__device__ __forceinline__ void head_pick_bin(const unsigned* lh, unsigned want, unsigned* part, unsigned* pick) {
  const int t = threadIdx.x;
  const unsigned a1 = lh[2047 - 2 * t], a0 = lh[2046 - 2 * t];
  const unsigned above = block_scan_u32(a1 + a0, part);
  if (above < want && want <= above + a1) { pick[0] = 2047 - 2 * t; pick[1] = want - above; }
  else if (above + a1 < want && want <= above + a1 + a0) { pick[0] = 2046 - 2 * t; pick[1] = want - above - a1; }
  __syncthreads();
}

// POOL: src_scores is the unpooled, non-negative metric; the clipped max-pool (half width
// sg.pool_kernel / 2; HALF = 3 is the compiled-in form of kernel 7, HALF < 0 the general one)
// and the forced +inf run here; pooled_out (may be NULL) receives the pooled scores.
// alloc_here: this workgroup also computes the budgets of its allocation problem (small form,
// one problem in the call; every head's workgroup does so for itself, the first one writes them).
template <bool POOL, int HALF>
__global__ __launch_bounds__(1024) void sel_head_kernel(SelGeom sg, SeqTab tab, AllocIO aio, int alloc_here,
                                                        const float* src_scores,
                                                        float* pooled_out, const int32_t* budgets,
                                                        int64_t* offsets_out, int n_heads_total,
                                                        unsigned* keepmask, unsigned* runpre,
                                                        unsigned* head_flag, int32_t* status) {
  extern __shared__ __align__(16) char smem[];
  float* stage = reinterpret_cast<float*>(smem) + kHeadRunLds;                       // run r at stage + 33 r
  unsigned* lh = reinterpret_cast<unsigned*>(smem + kHeadStageWords * 4);            // kHistBins
  unsigned* part = lh + kHistBins;                                                   // 16
  unsigned* pick = part + 16;                                                        // 4
  long long* osum = reinterpret_cast<long long*>(pick + 4);                          // 16
  int32_t* bud = reinterpret_cast<int32_t*>(osum + 16);                              // 64 (alloc_here)
  const int hi = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int kvh = hi % sg.n_kv_heads, layer = (hi / sg.n_kv_heads) % sg.n_layers;
  const int seq = hi / (sg.n_kv_heads * sg.n_layers);
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0, P = L - sg.window;
  const int64_t base = ((int64_t)layer * sg.n_kv_heads + kvh) * sg.total_tokens + tok0;
  const float* src = src_scores + base;
  // the selection status word starts at zero; the gather kernel ORs the heads' flags into it
  if (hi == 0 && t == 0) *status = 0;

  // scores through LDS: coalesced loads, all in flight together
  {
    const int n_in = POOL ? P : L;
    float v[kHeadRun];
#pragma unroll
    for (int u = 0; u < kHeadRun; ++u) {
      const int j = t + 1024 * u;
      v[u] = j < n_in ? src[j] : -INFINITY;
    }
    if (t < kHeadRunLds) { stage[t - kHeadRunLds] = -INFINITY; stage[1024 * kHeadRunLds + t] = -INFINITY; }
    lh[t] = 0;
    lh[t + 1024] = 0;
#pragma unroll
    for (int u = 0; u < kHeadRun; ++u) {
      const int j = t + 1024 * u;
      stage[(j >> 5) * kHeadRunLds + (j & 31)] = v[u];
    }
  }
  // inputs of the budget phase, in flight while the scores are processed
  AllocSmallLoad a_ld;
  if (alloc_here) a_ld = alloc_small_load(aio, seq);
  int kb = alloc_here ? 0 : budgets[hi];
  long long acc = 0;
  if (offsets_out && !alloc_here) {
    const int heads_per_seq = sg.n_kv_heads * sg.n_layers;
    for (int h2 = t; h2 < hi; h2 += 1024) {
      const int s2 = h2 / heads_per_seq, L2 = tab.cu[s2 + 1] - tab.cu[s2], b2 = budgets[h2];
      acc += b2 < 0 ? 0 : (b2 > L2 ? L2 : b2);
    }
  }
  __syncthreads();

  // this thread's run: pooled scores -> keys (registers).  Positions at or beyond L get key 0,
  // below every real key; `plain` threads hold 32 real, finite keys.
  const int j0 = kHeadRun * t;
  const int n_valid = L - j0 < 0 ? 0 : (L - j0 > kHeadRun ? kHeadRun : L - j0);
  const unsigned valid = n_valid == kHeadRun ? 0xFFFFFFFFu : ((1u << n_valid) - 1u);
  unsigned key[kHeadRun];
  unsigned fin = valid;               // real keys that are finite (they define the range)
  {
    const float* my = stage + t * kHeadRunLds;
    float s[kHeadRun];
    if (POOL) {
      if (HALF == 3) {
        float x[kHeadRun + 6];
        x[0] = my[-4]; x[1] = my[-3]; x[2] = my[-2];                       // the run before: its last three
#pragma unroll
        for (int i = 0; i < kHeadRun; ++i) x[3 + i] = my[i];
        x[35] = my[33]; x[36] = my[34]; x[37] = my[35];                    // the run after: its first three
#pragma unroll
        for (int i = 0; i < kHeadRun + 5; ++i) x[i] = fmaxf(x[i], x[i + 1]);          // 2 wide
#pragma unroll
        for (int i = 0; i < kHeadRun + 3; ++i) x[i] = fmaxf(x[i], x[i + 2]);          // 4 wide
#pragma unroll
        for (int i = 0; i < kHeadRun; ++i) s[i] = fmaxf(x[i], x[i + 3]);              // 7 wide
      } else {
        const int h = sg.pool_kernel >> 1;
#pragma unroll
        for (int i = 0; i < kHeadRun; ++i) {
          const int j = j0 + i;
          float m = -INFINITY;
          for (int p = max(0, j - h); p <= min(P - 1, j + h); ++p) m = fmaxf(m, stage[(p >> 5) * kHeadRunLds + (p & 31)]);
          s[i] = m;
        }
      }
      if (j0 < sg.n_sink || j0 + kHeadRun > P) {          // always kept (sink, observation window)
#pragma unroll
        for (int i = 0; i < kHeadRun; ++i) {
          const int j = j0 + i;
          if (j < sg.n_sink || j >= P) { s[i] = INFINITY; fin &= ~(1u << i); }
        }
      }
      if (pooled_out && n_valid) {
        float* dst = pooled_out + base + j0;
        if (n_valid == kHeadRun && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
#pragma unroll
          for (int i = 0; i < kHeadRun; i += 4)
            *reinterpret_cast<float4*>(dst + i) = make_float4(s[i], s[i + 1], s[i + 2], s[i + 3]);
        } else {
#pragma unroll
          for (int i = 0; i < kHeadRun; ++i)
            if (i < n_valid) dst[i] = s[i];
        }
      }
      // the metric is a sum of probabilities: non-negative, so its bits order like unsigned integers
#pragma unroll
      for (int i = 0; i < kHeadRun; ++i) key[i] = __float_as_uint(s[i]);
    } else {
#pragma unroll
      for (int i = 0; i < kHeadRun; ++i) {
        key[i] = key_of(my[i]);
        if (key[i] == 0xFF800000u || key[i] == 0x007FFFFFu) fin &= ~(1u << i);       // +inf, -inf
      }
    }
    if (n_valid != kHeadRun) {
#pragma unroll
      for (int i = 0; i < kHeadRun; ++i)
        if (i >= n_valid) key[i] = 0u;
    }
  }
  const bool plain = fin == 0xFFFFFFFFu;

  // range of the finite keys -> first digit scaled to it
  unsigned kmin = 0xFFFFFFFFu, kmax = 0u;
  if (plain) {
#pragma unroll
    for (int i = 0; i < kHeadRun; ++i) { kmin = umin_op(kmin, key[i]); kmax = umax_op(kmax, key[i]); }
  } else {
#pragma unroll
    for (int i = 0; i < kHeadRun; ++i)
      if ((fin >> i) & 1u) { kmin = umin_op(kmin, key[i]); kmax = umax_op(kmax, key[i]); }
  }
  if (offsets_out && !alloc_here) {
    if (wave * 64 < hi) {
#pragma unroll
      for (int o = 32; o > 0; o >>= 1) acc += shfl_xor_i64(acc, o);
    }
    if (lane == 0) osum[wave] = acc;
  }
  kmin = block_reduce_u32(kmin, 0xFFFFFFFFu, umin_op, part);
  kmax = block_reduce_u32(kmax, 0u, umax_op, part);
  unsigned lo = 0u, shift = 21u;        // no finite key: the top 11 bits of the key
  if (kmin <= kmax) {
    const unsigned span = kmax - kmin;
    const int bits = span ? 32 - __clz(span) : 0;
    lo = kmin;
    shift = bits > 11 ? (unsigned)(bits - 11) : 0u;
  }
  // first digit of every real key (the counters were cleared before the first barrier)
  if (valid == 0xFFFFFFFFu) {
#pragma unroll
    for (int i = 0; i < kHeadRun; ++i) atomicAdd(&lh[head_bin(key[i], lo, shift)], 1u);
  } else {
#pragma unroll
    for (int i = 0; i < kHeadRun; ++i)
      if (i < n_valid) atomicAdd(&lh[head_bin(key[i], lo, shift)], 1u);
  }
  // budgets: given, or computed here (the stage buffer is free now: every thread has its keys)
  if (alloc_here) {
    alloc_phase_b_small(aio, seq, smem, a_ld, bud, hi == 0);
    __syncthreads();
    kb = bud[hi];
    if (offsets_out && t == 0) {
      long long tot = 0;
      for (int h2 = 0; h2 < hi; ++h2) tot += bud[h2] < 0 ? 0 : (bud[h2] > L ? L : bud[h2]);
      offsets_out[hi] = tot;
      if (hi == n_heads_total - 1) offsets_out[n_heads_total] = tot + (kb < 0 ? 0 : (kb > L ? L : kb));
    }
  }
  unsigned flag = 0;
  if (kb < 0 || kb > L) { flag = LUKV_ST_CLAMPED; kb = kb < 0 ? 0 : L; }
  if (offsets_out && !alloc_here && t == 0) {
    long long tot = 0;
    for (int w2 = 0; w2 < 16; ++w2) tot += osum[w2];
    offsets_out[hi] = tot;
    if (hi == n_heads_total - 1) offsets_out[n_heads_total] = tot + kb;
  }
  const bool keep_none = kb == 0;       // runs the same code with k = 1 and overrides the result
  const unsigned k = keep_none ? 1u : (unsigned)kb;
  __syncthreads();                      // the histogram is complete
  head_pick_bin(lh, k, part, pick);
  const unsigned T0 = pick[0];
  unsigned want = pick[1];
  // the keys of bin T0 are the threshold candidates; digits over the bits in which they differ
  unsigned cand = 0;
  unsigned cmin = 0xFFFFFFFFu, cmax = 0u;
#pragma unroll
  for (int i = 0; i < kHeadRun; ++i) {
    const bool c = head_bin(key[i], lo, shift) == T0;
    cand |= c ? (1u << i) : 0u;
  }
  cand &= valid;
  if (cand) {
#pragma unroll
    for (int i = 0; i < kHeadRun; ++i)
      if ((cand >> i) & 1u) { cmin = umin_op(cmin, key[i]); cmax = umax_op(cmax, key[i]); }
  }
  cmin = block_reduce_u32(cmin, 0xFFFFFFFFu, umin_op, part);
  cmax = block_reduce_u32(cmax, 0u, umax_op, part);
  const unsigned span = cmax - cmin;
  int rest = span ? 32 - __clz(span) : 0;
  unsigned prefix = 0u;
  while (rest > 0) {
    const int sh = rest > 11 ? rest - 11 : 0;
    const unsigned mask = (1u << (rest - sh)) - 1u;
    lh[t] = 0;
    lh[t + 1024] = 0;
    __syncthreads();
    if (cand) {
#pragma unroll
      for (int i = 0; i < kHeadRun; ++i)
        if ((cand >> i) & 1u) atomicAdd(&lh[((key[i] - cmin) >> sh) & mask], 1u);
    }
    __syncthreads();
    head_pick_bin(lh, want, part, pick);
    const unsigned d = pick[0];
    want = pick[1];
    prefix |= d << sh;
    rest = sh;
    // only the keys with this digit stay candidates
    if (cand) {
      unsigned keep_c = 0;
#pragma unroll
      for (int i = 0; i < kHeadRun; ++i)
        keep_c |= (((cand >> i) & 1u) && (((key[i] - cmin) >> sh) & mask) == d) ? (1u << i) : 0u;
      cand = keep_c;
    }
    __syncthreads();      // pick and lh are rewritten by the next digit
  }
  const unsigned T = cmin + prefix;     // the k-th largest key; `want` of the keys equal to it are kept
  unsigned gt = 0, eq = 0;
#pragma unroll
  for (int i = 0; i < kHeadRun; ++i) {
    gt |= key[i] > T ? (1u << i) : 0u;
    eq |= key[i] == T ? (1u << i) : 0u;
  }
  gt &= valid;
  eq &= valid;
  // ties are kept in position order: this run's ties rank after those of the runs before it
  const unsigned n_eq = (unsigned)__popc(eq);
  const unsigned eq_before = block_scan_u32(n_eq, part);
  unsigned n_take = want > eq_before ? want - eq_before : 0u;
  n_take = n_take < n_eq ? n_take : n_eq;
  unsigned eq_keep = eq;
  for (unsigned n = n_eq; n > n_take; --n) eq_keep &= ~(0x80000000u >> __clz(eq_keep));   // drop the last tie
  const unsigned keep = keep_none ? 0u : (gt | eq_keep);
  const unsigned n_keep = (unsigned)__popc(keep);
  const unsigned before = block_scan_u32(n_keep, part);
  keepmask[(int64_t)hi * 1024 + t] = keep;
  runpre[(int64_t)hi * kHeadPrefixStride + t] = before;
  if (t == 1023) {
    runpre[(int64_t)hi * kHeadPrefixStride + 1024] = before + n_keep;
    head_flag[hi] = flag;
  }
}

// Gather for the whole-head selection: one workgroup per kGatherRuns runs (512 positions).  The
// keep masks and row prefixes of its runs give every kept position its output row; the positions
// go to kept_idx and the K and V rows are copied, 16 bytes per lane, eight rows in flight per
// thread.
constexpr int kGatherRuns = 16;
constexpr int kGatherElems = kGatherRuns * kHeadRun;   // 512 positions per workgroup

template <int ROW_BYTES>
__global__ __launch_bounds__(256) void sel_gather_kernel(SelGeom sg, SeqTab tab, const unsigned* keepmask,
                                                         const unsigned* runpre, const unsigned* head_flag,
                                                         const int64_t* offsets, const char* k,
                                                         const char* v, int64_t sl_bytes, int64_t sh_bytes,
                                                         int64_t st_bytes, int32_t* kept_idx, char* k_out,
                                                         char* v_out, int64_t out_rows, int32_t* status) {
  __shared__ int list[kGatherElems];
  int seq, blk;
  find_tile(tab, blockIdx.x, seq, blk);
  const int kvh = blockIdx.y, layer = blockIdx.z, t = threadIdx.x;
  const int tok0 = tab.cu[seq];
  const int hi = (seq * sg.n_layers + layer) * sg.n_kv_heads + kvh;
  constexpr int kPer = 256 / kGatherRuns;            // threads per run
  constexpr int kBits = kHeadRun / kPer;             // positions per thread
  const int run = blk * kGatherRuns + t / kPer, sub = t % kPer;
  const unsigned m = keepmask[(int64_t)hi * 1024 + run];
  const unsigned pre = runpre[(int64_t)hi * kHeadPrefixStride + run];
  const unsigned pre0 = runpre[(int64_t)hi * kHeadPrefixStride + blk * kGatherRuns];
  const unsigned pre1 = runpre[(int64_t)hi * kHeadPrefixStride + (blk + 1) * kGatherRuns];
  const int64_t head_row0 = offsets[hi];
  const unsigned flag = (blk == 0 && t == 0) ? head_flag[hi] : 0u;
  if (flag) atomicOr(status, (int)flag);
  unsigned n_keep = pre1 - pre0;
  {
    unsigned at = pre - pre0 + (unsigned)__popc(m & ((1u << (kBits * sub)) - 1u));
    const unsigned mine = (m >> (kBits * sub)) & ((1u << kBits) - 1u);
#pragma unroll
    for (int b = 0; b < kBits; ++b)
      if ((mine >> b) & 1u) list[at++] = run * kHeadRun + kBits * sub + b;
  }
  __syncthreads();
  // rows outside [0, out_rows) are dropped and flagged, never written; a head whose row offset is
  // negative (caller-supplied offsets) writes nothing at all
  const int64_t row0 = head_row0 + pre0;
  if (n_keep && (head_row0 < 0 || row0 + n_keep > out_rows)) {
    if (t == 0) atomicOr(status, LUKV_ST_CLAMPED);
    n_keep = head_row0 < 0 ? 0u : (row0 < out_rows ? (unsigned)(out_rows - row0) : 0u);
  }
  for (unsigned i = t; i < n_keep; i += 256) kept_idx[row0 + i] = list[i];
  constexpr int kLanesPerRow = ROW_BYTES / 16;
  constexpr int kRowsPerIter = 256 / kLanesPerRow;
  constexpr int kUnroll = 4;
  const int rsub = t / kLanesPerRow, col = (t % kLanesPerRow) * 16;
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
                        const uint4* state, const uint2* slice_cnt, const int64_t* offsets,
                        const void* k, const void* v, const Geom& g, int esize, int32_t* kept_idx,
                        void* k_out, void* v_out, int64_t out_rows, int32_t* status) {
  launch_staged(kStEmit, sel_emit_kernel<ROW_BYTES>, grid, dim3(256), st, sg, tab, pooled, state,
                slice_cnt, offsets, (const char*)k, (const char*)v, g.sl * esize, g.sh * esize,
                g.st * esize, kept_idx, (char*)k_out, (char*)v_out, out_rows, status);
}

template <int ROW_BYTES>
static void launch_gather(dim3 grid, hipStream_t st, SelGeom sg, const SeqTab& tab, const unsigned* keepmask,
                          const unsigned* runpre, const unsigned* head_flag, const int64_t* offsets,
                          const void* k, const void* v, const Geom& g, int esize, int32_t* kept_idx,
                          void* k_out, void* v_out, int64_t out_rows, int32_t* status) {
  launch_staged(kStGather, sel_gather_kernel<ROW_BYTES>, grid, dim3(256), st, sg, tab, keepmask, runpre,
                head_flag, offsets, (const char*)k, (const char*)v, g.sl * esize, g.sh * esize,
                g.st * esize, kept_idx, (char*)k_out, (char*)v_out, out_rows, status);
}

// the whole-head kernel needs more LDS than a kernel gets by default: raise its limit once
template <bool POOL, int HALF>
static bool head_kernel_ready() {
  static const bool ok = hipFuncSetAttribute(reinterpret_cast<const void*>(&sel_head_kernel<POOL, HALF>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize,
                                             kSelHeadLdsBytes) == hipSuccess;
  return ok;
}

template <bool POOL, int HALF>
static int launch_head(const HostCfg& hc, hipStream_t st, SelGeom sg, const SeqTab& tab, const AllocIO* aio,
                       const float* scores_in,
                       float* pooled_out, const int32_t* budgets, int64_t* offsets_out, unsigned* keepmask,
                       unsigned* runpre, unsigned* head_flag, int32_t* status) {
  if (!head_kernel_ready<POOL, HALF>()) { (void)hipGetLastError(); return LUKV_ELAUNCH; }
  AllocIO io;
  memset(&io, 0, sizeof(io));
  if (aio) io = *aio;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  stage_events(kStHead, &e0, &e1);
  hipExtLaunchKernelGGL((sel_head_kernel<POOL, HALF>), dim3(hc.n_hi), dim3(1024), kSelHeadLdsBytes, st, e0, e1, 0,
                        sg, tab, io, aio ? 1 : 0, scores_in, pooled_out, budgets, offsets_out, hc.n_hi, keepmask,
                        runpre, head_flag, status);
  return LUKV_OK;
}

// scores_in: pooled scores (pool = false) or the unpooled metric (pool = true; the pooled
// scores are then written to pooled_out, which may be NULL when every sequence takes the
// whole-head form, and used for the selection).
int launch_select_compact(const HostCfg& hc, const WsLayout& lay, const AllocIO* aio,
                          const float* scores_in, bool pool,
                          float* pooled_out, const int32_t* budgets, int64_t* offsets, bool make_offsets,
                          const void* k, const void* v, int32_t* kept_idx, void* k_out, void* v_out,
                          int64_t out_rows, int32_t* status, char* ws, hipStream_t st) {
  const Geom& g = hc.g;
  const int esize = g.f32 ? 4 : 2;
  const int row_bytes = g.head_dim * esize;
  if (row_bytes != 128 && row_bytes != 256 && row_bytes != 512) return LUKV_EDTYPE;
  const SeqTab tabH = tiles_for(hc.seq, kSliceElems, 0);
  SelGeom sg{g.n_layers, g.n_kv_heads, g.total_tokens, lay.max_slices,
             g.window, g.pool_kernel, g.n_sink,
             pool ? g.chunk_keys : kSliceElems, pool ? 4 : 1, pool ? g.window : 0,
             pool ? lay.max_chunks * 4 : lay.max_slices, 1};
  if (select_whole_head(hc)) {
    // two kernels: one workgroup per head decides, then the gather
    unsigned* keepmask = reinterpret_cast<unsigned*>(ws + lay.keepmask);
    unsigned* runpre = reinterpret_cast<unsigned*>(ws + lay.runpre);
    unsigned* head_flag = reinterpret_cast<unsigned*>(ws + lay.head_flag);
    int64_t* off_out = make_offsets ? offsets : (int64_t*)nullptr;
    int rc;
    // aio here means: the budgets are computed by the head workgroups themselves (small form)
    if (!pool) rc = launch_head<false, -1>(hc, st, sg, tabH, aio, scores_in, nullptr, budgets, off_out, keepmask, runpre, head_flag, status);
    else if (g.pool_kernel == 7) rc = launch_head<true, 3>(hc, st, sg, tabH, aio, scores_in, pooled_out, budgets, off_out, keepmask, runpre, head_flag, status);
    else rc = launch_head<true, -1>(hc, st, sg, tabH, aio, scores_in, pooled_out, budgets, off_out, keepmask, runpre, head_flag, status);
    if (rc) return rc;
    const SeqTab tabG = tiles_for(hc.seq, kGatherElems, 0);
    dim3 gridG(tabG.tile0[tabG.n_seqs], g.n_kv_heads, g.n_layers);
    if (row_bytes == 128)
      launch_gather<128>(gridG, st, sg, tabG, keepmask, runpre, head_flag, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
    else if (row_bytes == 256)
      launch_gather<256>(gridG, st, sg, tabG, keepmask, runpre, head_flag, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
    else
      launch_gather<512>(gridG, st, sg, tabG, keepmask, runpre, head_flag, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
    return check_launch();
  }
  const SeqTab tabE = tiles_for(hc.seq, kEmitElems, 0);
  // calls with thousands of slices: a few slices per histogram workgroup (thresholds in units
  // of the 1024-thread workgroups the chip holds at once, two per CU)
  {
    const int64_t n_slice_wgs = (int64_t)tabH.tile0[tabH.n_seqs] * g.n_kv_heads * g.n_layers;
    if (n_slice_wgs >= 4096) sg.slices_per_wg = 4;
    else if (n_slice_wgs >= 2048) sg.slices_per_wg = 2;
  }
  const SeqTab tabHW = tiles_for(hc.seq, kSliceElems * sg.slices_per_wg, 0);
  unsigned* hist = reinterpret_cast<unsigned*>(ws + lay.hist);
  float2* range = reinterpret_cast<float2*>(ws + lay.range);
  uint2* head_dig = reinterpret_cast<uint2*>(ws + lay.head_dig);
  uint4* state = reinterpret_cast<uint4*>(ws + lay.sel_state);
  uint2* slice_cnt = reinterpret_cast<uint2*>(ws + lay.slice_cnt);
  unsigned long long* by_bin = reinterpret_cast<unsigned long long*>(ws + lay.by_bin);
  unsigned long long* cand = reinterpret_cast<unsigned long long*>(ws + lay.cand);
  AllocIO io;
  memset(&io, 0, sizeof(io));
  int n_alloc = 0;
  if (aio) { io = *aio; n_alloc = aio->n_problems; }
  const int n_tiles = tabH.tile0[tabH.n_seqs];
  dim3 gridH(tabHW.tile0[tabHW.n_seqs] + n_alloc, g.n_kv_heads, g.n_layers);
  dim3 gridR(n_tiles, g.n_kv_heads, g.n_layers);
  dim3 gridE(tabE.tile0[tabE.n_seqs], g.n_kv_heads, g.n_layers);
  if (pool) {
    launch_staged(kStHist, sel_hist_kernel<true>, gridH, dim3(1024), st, sg, tabHW, io, n_alloc, scores_in,
                  pooled_out, (const float2*)range, hist, head_dig, by_bin, status);
  } else {
    hipLaunchKernelGGL(sel_range_kernel, gridR, dim3(1024), 0, st, sg, tabH, scores_in, range);
    launch_staged(kStHist, sel_hist_kernel<false>, gridH, dim3(1024), st, sg, tabHW, io, n_alloc, scores_in,
                  (float*)nullptr, (const float2*)range, hist, head_dig, by_bin, status);
  }
  const float* sel_scores = pool ? pooled_out : scores_in;
  launch_staged(kStTail, sel_tail_kernel, dim3(hc.n_hi), dim3(1024), st, sg, tabH, budgets,
                (const unsigned*)hist, (const unsigned long long*)by_bin, (const uint2*)head_dig, state, slice_cnt, cand,
                make_offsets ? offsets : (int64_t*)nullptr, hc.n_hi, status);
  if (row_bytes == 128)
    launch_emit<128>(gridE, st, sg, tabE, sel_scores, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else if (row_bytes == 256)
    launch_emit<256>(gridE, st, sg, tabE, sel_scores, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  else
    launch_emit<512>(gridE, st, sg, tabE, sel_scores, state, slice_cnt, offsets, k, v, g, esize, kept_idx, k_out, v_out, out_rows, status);
  return check_launch();
}

// The whole-head form takes about 20 us per head on one compute unit whatever the number of
// heads (a head's 32768 scores pass through one unit's ALUs and LDS), the per-slice form about
// 13 us plus 3 us per 8 heads: the former pays from a few dozen heads on.
bool select_whole_head(const HostCfg& hc) { return hc.max_len <= kSelHeadMaxLen && hc.n_hi >= 64; }

}  // namespace lukv
