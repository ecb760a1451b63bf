// Baseline allocation by a global top-k (Sec. 4.2 opening; Sec. 5.1 "Baselines"): the candidate
// positions of all heads of a sequence are pooled, the B_total of largest surrogate score are
// retained, and a head's budget is the number of its positions among them; with a floor, every
// head first keeps its `floor` best positions and only the rest compete.
//
// With c_h(x) = number of positions of head h that come before x in the pooled order (score
// descending, head ascending, position ascending), the budgets are b_h = max(floor, c_h(cut)) for
// the one cut at which they sum to B_total.  The cut is found by a most-significant-digit radix
// search over the 32-bit order-preserving keys of the scores, four digits of eight bits: per digit
// one pass over the scores builds a 256-bin histogram PER HEAD (only of the keys that share the
// digits fixed so far), then one workgroup per sequence sums max(floor, above_h + suffix_h(bin))
// over the heads for every bin and fixes the bin in which that sum reaches B_total.  After the
// last digit the cut's score is known exactly; positions of that score are handed out in head
// order until B_total is reached (their order inside a head is the selection's tie rule).
#include <string.h>

#include "lukv_internal.hpp"

namespace lukv {

constexpr int kTkBins = 256;      // bins per digit
constexpr int kTkDigits = 4;      // 4 x 8 bits = the whole key
constexpr int kTkSlice = 4096;    // positions one histogram workgroup reads
constexpr int kTkMaxHeads = 4096; // heads per sequence (the last step keeps two words per head in LDS)

struct TopkArgs {
  int32_t n_heads;                  // heads per sequence: n_layers * n_kv_heads
  int32_t floor;                    // places every head keeps whatever its scores
  int32_t total_tokens;
  int64_t B[LUKV_MAX_SEQS];
  int32_t mode[LUKV_MAX_SEQS];      // decided on the host: 0 infeasible, 1 search, 2 every head at its floor
                                    // (feasible: floor <= L, n_heads * floor <= B <= n_heads * L)
  unsigned* hist;                   // [n_seqs][n_heads][256]
  unsigned* above;                  // [n_seqs][n_heads] positions before the range still searched
  unsigned* prefix;                 // [n_seqs] digits fixed so far
};

// order-preserving key of a score: larger score = larger key; -0 and +0 share a key
__device__ __forceinline__ unsigned topk_key(float x) {
  const unsigned u = __float_as_uint(x + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ __launch_bounds__(256) void topk_clear_kernel(TopkArgs a, int n_seqs) {
  const int64_t n_hist = (int64_t)n_seqs * a.n_heads * kTkBins;
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_hist) a.hist[i] = 0u;
  if (i < (int64_t)n_seqs * a.n_heads) a.above[i] = 0u;
  if (i < n_seqs) a.prefix[i] = 0u;
}

// digit `pass` (0 = most significant) of the keys that carry the digits fixed so far
__global__ __launch_bounds__(256) void topk_hist_kernel(TopkArgs a, SeqTab tab, const float* scores, int pass) {
  __shared__ unsigned bins[kTkBins];
  int seq, tile;
  find_tile(tab, blockIdx.x, seq, tile);
  if (a.mode[seq] != 1) return;
  const int h = blockIdx.y;
  const int tok0 = tab.cu[seq], L = tab.cu[seq + 1] - tok0;
  bins[threadIdx.x] = 0u;
  __syncthreads();
  const unsigned prefix = a.prefix[seq];
  const int shift = 24 - 8 * pass;
  const float* src = scores + (int64_t)h * a.total_tokens + tok0;
  const int j0 = tile * kTkSlice;
#pragma unroll 4
  for (int it = 0; it < kTkSlice / 256; ++it) {
    const int j = j0 + it * 256 + (int)threadIdx.x;
    if (j < L) {
      const unsigned key = topk_key(src[j]);
      // (a 32-bit shift by 32 is undefined: the first pass takes every key)
      if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&bins[(key >> shift) & 255u], 1u);
    }
  }
  __syncthreads();
  const unsigned c = bins[threadIdx.x];
  if (c) atomicAdd(&a.hist[((int64_t)seq * a.n_heads + h) * kTkBins + threadIdx.x], c);
}

__device__ __forceinline__ unsigned long long topk_block_sum(unsigned long long v, unsigned long long* part) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
  __syncthreads();
  unsigned long long s = 0;
  for (int w = 0; w < 16; ++w) s += part[w];
  return s;
}

// exclusive prefix sum over the 1024 threads (thread order), total in *tot
__device__ __forceinline__ unsigned long long topk_block_scan(unsigned long long v, unsigned long long* part,
                                                              unsigned long long* tot) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long incl = v;
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long up = __shfl_up(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) part[wave] = incl;
  __syncthreads();
  unsigned long long before = 0, all = 0;
  for (int w = 0; w < 16; ++w) {
    const unsigned long long t = part[w];
    if (w < wave) before += t;
    all += t;
  }
  *tot = all;
  return before + incl - v;
}

// One workgroup per sequence: fixes digit `pass`; after the last digit writes the budgets.
__global__ __launch_bounds__(1024) void topk_decide_kernel(TopkArgs a, int pass, int32_t* budgets, int32_t* status) {
  // 32 KiB: first the per-wave sums of every bin, then (last digit) two words per head
  __shared__ __align__(16) unsigned long long buf[16 * kTkBins];
  __shared__ unsigned long long part[16];
  __shared__ unsigned long long s_incl[kTkBins + 1];
  __shared__ int s_bin;
  const int seq = blockIdx.x, NH = a.n_heads;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool last = pass == kTkDigits - 1;
  int32_t* b_out = budgets + (int64_t)seq * NH;
  if (a.mode[seq] != 1) {          // uniform over the workgroup
    if (last) {
      for (int h = threadIdx.x; h < NH; h += 1024) b_out[h] = a.floor;
      if (threadIdx.x == 0) status[seq] = a.mode[seq] == 0 ? LUKV_ST_INFEASIBLE : 0;
    }
    return;
  }
  const unsigned long long B = (unsigned long long)a.B[seq];
  const unsigned fl = (unsigned)a.floor;
  u32x4* H4 = reinterpret_cast<u32x4*>(a.hist + (int64_t)seq * NH * kTkBins);
  unsigned* above = a.above + (int64_t)seq * NH;

  // sum over the heads of max(floor, above_h + positions of head h in bins >= b), for every bin b:
  // a wave takes every 16th head, a lane four neighbouring bins
  unsigned long long acc[4] = {0, 0, 0, 0};
  unsigned long long excl = 0;      // the same sum with no bin of this digit included
  for (int h = wave; h < NH; h += 16) {
    const u32x4 c = H4[(int64_t)h * 64 + lane];
    const unsigned t = c.x + c.y + c.z + c.w;
    const unsigned incl = wave_scan_incl(t);
    const unsigned after = (unsigned)__builtin_amdgcn_readlane((int)incl, 63) - incl;   // bins of higher lanes
    const unsigned ab = above[h];
    const unsigned s3 = after + c.w, s2 = s3 + c.z, s1 = s2 + c.y, s0 = s1 + c.x;
    acc[0] += max(fl, ab + s0);
    acc[1] += max(fl, ab + s1);
    acc[2] += max(fl, ab + s2);
    acc[3] += max(fl, ab + s3);
    if (lane == 0) excl += max(fl, ab);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) buf[wave * kTkBins + 4 * lane + i] = acc[i];
  excl = topk_block_sum(excl, part);      // (two barriers: buf is complete after it)
  if (threadIdx.x < kTkBins) {
    unsigned long long s = 0;
    for (int w = 0; w < 16; ++w) s += buf[w * kTkBins + threadIdx.x];
    s_incl[threadIdx.x] = s;
  }
  if (threadIdx.x == 0) {
    s_incl[kTkBins] = excl;
    s_bin = 0;
  }
  __syncthreads();
  // the sums do not increase with the bin: exactly one bin reaches B while the next one does not
  if (threadIdx.x < kTkBins && s_incl[threadIdx.x] >= B && s_incl[threadIdx.x + 1] < B) s_bin = threadIdx.x;
  __syncthreads();
  const int bin = s_bin;

  // positions above the chosen bin join `above`; the histogram is left cleared for the next digit
  unsigned* ab_l = reinterpret_cast<unsigned*>(buf);          // [NH] (last digit)
  unsigned* eq_l = ab_l + kTkMaxHeads;                        // [NH] positions in the chosen bin
  for (int h = wave; h < NH; h += 16) {
    const u32x4 c = H4[(int64_t)h * 64 + lane];
    const int b0 = 4 * lane;
    unsigned gt = (b0 > bin ? c.x : 0u) + (b0 + 1 > bin ? c.y : 0u) + (b0 + 2 > bin ? c.z : 0u) + (b0 + 3 > bin ? c.w : 0u);
    unsigned eq = b0 == bin ? c.x : b0 + 1 == bin ? c.y : b0 + 2 == bin ? c.z : b0 + 3 == bin ? c.w : 0u;
    gt = wave_scan_incl(gt);
    eq = wave_scan_incl(eq);
    H4[(int64_t)h * 64 + lane] = u32x4{0u, 0u, 0u, 0u};
    if (lane == 63) {
      const unsigned ab = above[h] + gt;
      above[h] = ab;
      if (last) {
        ab_l[h] = ab;
        eq_l[h] = eq;
      }
    }
  }
  if (threadIdx.x == 0) a.prefix[seq] = (a.prefix[seq] << 8) | (unsigned)bin;
  if (!last) return;
  __syncthreads();

  // The cut's score is known.  Every head keeps max(floor, above_h); what is still missing goes
  // to the positions of exactly that score, head by head in ascending order.
  unsigned long long base_sum = 0;
  for (int h = threadIdx.x; h < NH; h += 1024) base_sum += max(fl, ab_l[h]);
  base_sum = topk_block_sum(base_sum, part);
  const unsigned long long need = B - base_sum;        // > 0: the sum without the bin stays below B
  unsigned long long carry = 0;
  for (int h0 = 0; h0 < NH; h0 += 1024) {
    const int h = h0 + (int)threadIdx.x;
    unsigned base = 0, gain = 0;
    if (h < NH) {
      base = max(fl, ab_l[h]);
      gain = max(fl, ab_l[h] + eq_l[h]) - base;
    }
    unsigned long long tot;
    const unsigned long long before = carry + topk_block_scan(gain, part, &tot);
    if (h < NH) {
      unsigned long long b = base;
      if (before + gain <= need) b += gain;
      else if (before < need) b += need - before;
      b_out[h] = (int32_t)b;
    }
    carry += tot;
  }
  if (threadIdx.x == 0) status[seq] = 0;
}

int64_t topk_workspace_bytes(int32_t n_seqs, int32_t n_heads) {
  return (int64_t)n_seqs * n_heads * (kTkBins * 4 + 4) + (int64_t)n_seqs * 4 + 512;
}

int launch_allocate_topk(const HostCfg& hc, const float* scores, const int64_t* B_total, int32_t floor,
                         int32_t* budgets, int64_t* offsets, int32_t* status, char* ws, hipStream_t st) {
  const int n_seqs = hc.seq.n_seqs, NH = hc.g.n_layers * hc.g.n_kv_heads;   // heads per sequence
  if (NH > kTkMaxHeads) return LUKV_EINVAL;
  TopkArgs a;
  memset(&a, 0, sizeof(a));
  a.n_heads = NH;
  a.floor = floor;
  a.total_tokens = hc.g.total_tokens;
  for (int s = 0; s < n_seqs; ++s) {
    const int64_t L = hc.seq.cu[s + 1] - hc.seq.cu[s];
    a.B[s] = B_total[s];
    const bool ok = floor >= 0 && floor <= L && B_total[s] >= (int64_t)NH * floor && B_total[s] <= (int64_t)NH * L;
    // (with no place beyond the floors there is no cut to search for)
    a.mode[s] = !ok ? 0 : B_total[s] == (int64_t)NH * floor ? 2 : 1;
  }
  a.hist = reinterpret_cast<unsigned*>(ws);
  a.above = a.hist + (int64_t)n_seqs * NH * kTkBins;
  a.prefix = a.above + (int64_t)n_seqs * NH;
  const int64_t n_hist = (int64_t)n_seqs * NH * kTkBins;
  hipLaunchKernelGGL(topk_clear_kernel, dim3((unsigned)((n_hist + 255) / 256)), dim3(256), 0, st, a, n_seqs);
  const SeqTab tab = tiles_for(hc.seq, kTkSlice, 0);
  for (int pass = 0; pass < kTkDigits; ++pass) {
    hipLaunchKernelGGL(topk_hist_kernel, dim3(tab.tile0[tab.n_seqs], NH), dim3(256), 0, st, a, tab, scores, pass);
    hipLaunchKernelGGL(topk_decide_kernel, dim3(n_seqs), dim3(1024), 0, st, a, pass, budgets, status);
  }
  launch_offsets(budgets, offsets, (int64_t)n_seqs * NH, st);
  return check_launch();
}

}  // namespace lukv
