// Step 2: global head-level budget allocation (Sec. 4.2 "Efficient Optimization via Convex
// Hull Relaxation", Eq. 8-10; App. A.2 "Optimality of greedy allocation").
//
// The unit-by-unit greedy of the paper picks, B times, the head whose next unit has the
// largest marginal gain.  Gains are constant along a hull segment and strictly decreasing
// from one segment of a head to the next, so the greedy result is a weighted selection:
// find the gain g* at which the cumulated units (largest gain first) reach the remaining
// budget, give every head all its units above g*, and hand the units at exactly g* out in
// head order.  One workgroup per problem:
//   1. one thread per head: monotone-chain upper hull of (knot, U), segments clipped to
//      (b_min, min(b_max, last knot)] with their gain as an order-preserving 64-bit key;
//   2. weighted radix select (8 digits of 8 bits, LDS histogram of unit counts) for g*;
//   3. budgets per head, ties by a prefix sum over heads;
//   4. the last problem to finish writes the exclusive prefix sum of all budgets (offsets).
//
// This file is compiled with -ffp-contract=off: a gain is one fp64 subtract and one fp64
// divide, nothing fused, so that it compares bit for bit like the same expression on a CPU.
#include "lukv_internal.hpp"

namespace lukv {

__device__ __forceinline__ double gain(const float* U, const int32_t* n, int a, int b) {
  return ((double)U[b] - (double)U[a]) / (double)(n[b] - n[a]);
}

__device__ __forceinline__ unsigned long long gain_key(double x) {
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  if (x == 0.0) u = 0ull;  // -0 and +0 tie
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

// exclusive scan of one int64 per thread over the 256 threads; sm has 256 slots
__device__ long long block_scan(long long v, long long* sm, long long* total) {
  const int t = threadIdx.x;
  __syncthreads();
  sm[t] = v;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const long long add = t >= o ? sm[t - o] : 0;
    __syncthreads();
    sm[t] += add;
    __syncthreads();
  }
  const long long incl = sm[t];
  *total = sm[255];
  return incl - v;
}

struct AllocArgs {
  int32_t n_problems, n_heads, n_grid;
  int64_t B[LUKV_MAX_SEQS];
};

__global__ __launch_bounds__(256) void allocate_kernel(AllocArgs aa, const float* curves,
                                                       const int32_t* knots, const int32_t* b_min,
                                                       const int32_t* b_max, int32_t* budgets,
                                                       int64_t* offsets, int32_t* status,
                                                       int32_t* hull, unsigned long long* seg_key,
                                                       unsigned* seg_w, unsigned* counter) {
  __shared__ long long sm[256];
  __shared__ unsigned long long hist[256];
  __shared__ unsigned long long sel_prefix;
  __shared__ long long sel_rem;
  __shared__ int is_last;
  const int p = blockIdx.x, NH = aa.n_heads, Gp = aa.n_grid, t = threadIdx.x;
  const int64_t hbase = (int64_t)p * NH;
  const int64_t nseg = (int64_t)NH * Gp;
  unsigned long long* skey = seg_key + hbase * Gp;
  unsigned* sw = seg_w + hbase * Gp;

  // 1. hulls and clipped segments
  long long sum_min = 0, sum_w = 0;
  int bad = 0;
  for (int h = t; h < NH; h += 256) {
    const float* U = curves + (hbase + h) * Gp;
    const int32_t* n = knots + (hbase + h) * Gp;
    int32_t* stck = hull + (hbase + h) * Gp;
    int top = 0;
    for (int g = 0; g < Gp; ++g) {
      stck[top++] = g;
      while (top >= 3 &&
             gain(U, n, stck[top - 3], stck[top - 2]) <= gain(U, n, stck[top - 2], stck[top - 1])) {
        stck[top - 2] = stck[top - 1];
        --top;
      }
    }
    const long long lo_b = b_min[hbase + h];
    const long long cap = min((long long)b_max[hbase + h], (long long)n[Gp - 1]);
    if (lo_b < 0 || lo_b > cap) bad = 1;
    sum_min += lo_b;
    for (int e = 0; e < Gp; ++e) {
      unsigned w = 0;
      unsigned long long key = 0;
      if (e + 1 < top) {
        const int a = stck[e], b = stck[e + 1];
        const long long lo = max((long long)n[a], lo_b), hi = min((long long)n[b], cap);
        w = hi > lo ? (unsigned)(hi - lo) : 0u;
        key = gain_key(gain(U, n, a, b));
      }
      skey[(int64_t)h * Gp + e] = key;
      sw[(int64_t)h * Gp + e] = w;
      sum_w += w;
    }
  }
  long long tot_min, tot_w, tot_bad;
  block_scan(sum_min, sm, &tot_min);
  block_scan(sum_w, sm, &tot_w);
  block_scan(bad, sm, &tot_bad);
  const long long R = aa.B[p] - tot_min;
  const bool infeasible = tot_bad != 0 || R < 0 || R > tot_w;
  __syncthreads();  // segment arrays written above are read by other threads below

  // 2. weighted radix select of the threshold gain g*: W(> g*) < R <= W(>= g*)
  if (t == 0) { sel_prefix = 0ull; sel_rem = R; }
  __syncthreads();
  if (!infeasible && R > 0) {
    for (int shift = 56; shift >= 0; shift -= 8) {
      hist[t] = 0ull;
      __syncthreads();
      const unsigned long long prefix = sel_prefix;
      for (int64_t i = t; i < nseg; i += 256) {
        const unsigned w = sw[i];
        if (w) {
          const unsigned long long key = skey[i];
          if (shift == 56 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
            atomicAdd(&hist[(key >> shift) & 255ull], (unsigned long long)w);
        }
      }
      __syncthreads();
      // thread t owns descending bin t
      const long long mine = (long long)hist[255 - t];
      long long dummy;
      const long long before = block_scan(mine, sm, &dummy);
      const long long want = sel_rem;
      __syncthreads();
      if (before < want && want <= before + mine) {
        sel_prefix = prefix | ((unsigned long long)(255 - t) << shift);
        sel_rem = want - before;
      }
      __syncthreads();
    }
  }
  const unsigned long long kstar = sel_prefix;
  const long long rem = (!infeasible && R > 0) ? sel_rem : 0;

  // 3. budgets: everything above g*, ties at g* in head order
  long long carry = 0;
  for (int h0 = 0; h0 < NH; h0 += 256) {
    const int h = h0 + t;
    long long gt = 0, eq = 0;
    if (h < NH && !infeasible && R > 0) {
      for (int e = 0; e < Gp; ++e) {
        const unsigned w = sw[(int64_t)h * Gp + e];
        const unsigned long long key = skey[(int64_t)h * Gp + e];
        if (key > kstar) gt += w;
        else if (key == kstar) eq += w;
      }
    }
    long long tot;
    const long long eq_before = carry + block_scan(eq, sm, &tot);
    carry += tot;
    if (h < NH) {
      long long take = rem - eq_before;
      take = take < 0 ? 0 : (take > eq ? eq : take);
      budgets[hbase + h] = (int32_t)(b_min[hbase + h] + gt + take);
    }
  }
  if (t == 0) status[p] = infeasible ? LUKV_ST_INFEASIBLE : 0;

  // 4. offsets over all problems, by the last workgroup to get here
  __threadfence();
  __syncthreads();
  if (t == 0) is_last = atomicAdd(counter, 1u) == (unsigned)(aa.n_problems - 1);
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  const int64_t n_all = (int64_t)aa.n_problems * NH;
  long long run = 0;
  for (int64_t i0 = 0; i0 < n_all; i0 += 256) {
    const int64_t i = i0 + t;
    const long long b = i < n_all ? (long long)__builtin_nontemporal_load(&budgets[i]) : 0;
    long long tot;
    const long long ex = run + block_scan(b, sm, &tot);
    if (i < n_all) offsets[i] = ex;
    run += tot;
  }
  if (t == 0) offsets[n_all] = run;
}

int launch_allocate(int32_t n_problems, int32_t n_heads, int32_t n_grid, const float* curves,
                    const int32_t* knots, const int32_t* b_min, const int32_t* b_max,
                    const int64_t* B_total, int32_t* budgets, int64_t* offsets, int32_t* status,
                    const WsLayout& lay, char* ws, hipStream_t st) {
  AllocArgs aa;
  aa.n_problems = n_problems;
  aa.n_heads = n_heads;
  aa.n_grid = n_grid;
  for (int i = 0; i < LUKV_MAX_SEQS; ++i) aa.B[i] = i < n_problems ? B_total[i] : 0;
  stage_mark(kStAllocate, st);
  hipLaunchKernelGGL(allocate_kernel, dim3(n_problems), dim3(256), 0, st, aa, curves, knots, b_min,
                     b_max, budgets, offsets, status, reinterpret_cast<int32_t*>(ws + lay.hull),
                     reinterpret_cast<unsigned long long*>(ws + lay.seg_key),
                     reinterpret_cast<unsigned*>(ws + lay.seg_w),
                     reinterpret_cast<unsigned*>(ws + lay.alloc_cnt));
  return check_launch();
}

}  // namespace lukv
