// Device code of step 2, the global head-level budget allocation (Sec. 4.2 "Efficient
// Optimization via Convex Hull Relaxation", Eq. 8-10; App. A.2 "Optimality of greedy
// allocation"), written for a 256-thread workgroup per problem so that it can run either
// in its own kernel or as one extra workgroup of a score kernel.
//
// The unit-by-unit greedy of the paper picks, B times, the head whose next unit has the
// largest marginal gain.  Gains are constant along a hull segment and strictly decreasing
// from one segment of a head to the next, so the greedy result is a weighted selection:
// find the gain g* at which the cumulated units (largest gain first) reach the remaining
// budget, give every head all its units above g*, and hand the units at exactly g* out in
// head order.
//   phase A: one thread per (head, knot): hull vertices by the chord criterion; hull segments
//            clipped to (b_min, min(b_max, last knot)] with their gain as an order-preserving
//            64-bit key; per-problem sums for the feasibility check.
//   phase B: weighted radix select (8 digits of 8 bits, LDS histogram of unit counts) for
//            g*; budgets per head (ties by a prefix sum over heads).  The row offsets
//            (prefix sum of all budgets) are written by whoever consumes the budgets next.
//
// Nothing here may be fused: a gain is one fp64 subtract and one fp64 divide, so that it
// compares bit for bit like the same expression evaluated on a CPU.
#pragma once

#include "lukv_internal.hpp"

#pragma clang fp contract(off)

namespace lukv {

struct AllocIO {
  int32_t n_problems, n_heads, n_grid;
  const float* curves;
  const int32_t* knots;
  const int32_t* b_min;
  const int32_t* b_max;
  int32_t* budgets;
  int64_t* offsets;
  int32_t* status;
  unsigned long long* seg_key;  // [n_problems * n_heads * n_grid]
  unsigned* seg_w;              // same
  long long* meta;              // [n_problems * 4]: sum b_min, sum units, bad flag
  int64_t B[LUKV_MAX_SEQS];
};

struct HullPoint {
  int32_t n;
  float U;
};

__device__ __forceinline__ unsigned long long gain_key(double x) {
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  if (x == 0.0) u = 0ull;  // -0 and +0 tie
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ long long shfl_up_i64(long long v, int o) {
  int lo = __shfl_up((int)(v & 0xFFFFFFFFll), o), hi = __shfl_up((int)(v >> 32), o);
  return ((long long)hi << 32) | (unsigned)lo;
}

// Exclusive scan of one int64 per thread over 256 threads (4 waves); sm has >= 4 slots.
__device__ __forceinline__ long long block_scan_i64(long long v, long long* sm, long long* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  long long incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const long long up = shfl_up_i64(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) sm[wave] = incl;
  __syncthreads();
  long long before = 0;
  for (int w = 0; w < wave; ++w) before += sm[w];
  *total = sm[0] + sm[1] + sm[2] + sm[3];
  return before + incl - v;
}

// Phase A for problem p.  lds: scratch of lds_bytes (>= 32 KiB), free for this call.
// Hull vertices by their definition, one (head, knot) pair per thread: knot g is a vertex of
// the upper concave hull iff every chord from an earlier knot to g is strictly steeper than
// every chord from g to a later knot (end knots always are).  All chords are independent
// fp64 divisions, so nothing here waits on a serial chain; consecutive vertices then give
// the segments, whose gains are strictly decreasing by the same criterion.
__device__ inline void alloc_phase_a(const AllocIO& io, int p, char* lds, int lds_bytes) {
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x;
  const int64_t hbase = (int64_t)p * NH;
  long long* sm = reinterpret_cast<long long*>(lds);          // 4 slots
  HullPoint* pts = reinterpret_cast<HullPoint*>(lds + 64);
  int heads_per_batch = (lds_bytes - 64) / (int)((sizeof(HullPoint) + sizeof(int)) * Gp);
  heads_per_batch = heads_per_batch > NH ? NH : heads_per_batch;
  int* vertex = reinterpret_cast<int*>(lds + 64 + (int64_t)heads_per_batch * Gp * sizeof(HullPoint));
  long long sum_min = 0, sum_w = 0, bad = 0;
  if (heads_per_batch < 1) bad = 1;  // curve too long for the scratch: flagged, never run
  for (int h0 = 0; h0 < NH && heads_per_batch >= 1; h0 += heads_per_batch) {
    const int nb = min(heads_per_batch, NH - h0);
    const int64_t gbase = (hbase + h0) * Gp;
    __syncthreads();
    for (int i = t; i < nb * Gp; i += 256) {
      HullPoint e;
      e.n = io.knots[gbase + i];
      e.U = io.curves[gbase + i];
      pts[i] = e;
    }
    __syncthreads();
    for (int i = t; i < nb * Gp; i += 256) {
      const int hh = i / Gp, g = i - hh * Gp;
      const HullPoint* ph = pts + hh * Gp;
      const HullPoint me = ph[g];
      int is_vertex = 1;
      if (g > 0 && g < Gp - 1) {
        double steep_in = INFINITY, steep_out = -INFINITY;
        // independent divisions: unrolled so that several are in flight (one fp64 division
        // is a long dependent chain of its own)
#pragma unroll 8
        for (int a = 0; a < g; ++a) {
          const HullPoint o = ph[a];
          const double s = ((double)me.U - (double)o.U) / (double)(me.n - o.n);
          steep_in = s < steep_in ? s : steep_in;
        }
#pragma unroll 8
        for (int c = g + 1; c < Gp; ++c) {
          const HullPoint o = ph[c];
          const double s = ((double)o.U - (double)me.U) / (double)(o.n - me.n);
          steep_out = s > steep_out ? s : steep_out;
        }
        is_vertex = steep_in > steep_out;
      }
      vertex[i] = is_vertex;
    }
    __syncthreads();
    // one segment per vertex (to the next vertex), clipped to (b_min, cap], stored coalesced
    for (int i = t; i < nb * Gp; i += 256) {
      const int hh = i / Gp, g = i - hh * Gp;
      const HullPoint* ph = pts + hh * Gp;
      const long long lb = io.b_min[hbase + h0 + hh];
      const long long cp = min((long long)io.b_max[hbase + h0 + hh], (long long)ph[Gp - 1].n);
      if (g == 0) {
        if (lb < 0 || lb > cp) bad = 1;
        sum_min += lb;
      }
      unsigned w = 0;
      unsigned long long key = 0;
      if (vertex[i] && g < Gp - 1) {
        int c = g + 1;
        while (!vertex[hh * Gp + c]) ++c;   // the last knot is always a vertex
        const HullPoint a = ph[g], b = ph[c];
        const long long lo = max((long long)a.n, lb), hi = min((long long)b.n, cp);
        w = hi > lo ? (unsigned)(hi - lo) : 0u;
        key = gain_key(((double)b.U - (double)a.U) / (double)(b.n - a.n));
      }
      io.seg_key[gbase + i] = key;
      io.seg_w[gbase + i] = w;
      sum_w += w;
    }
  }
  long long tot_min, tot_w, tot_bad;
  block_scan_i64(sum_min, sm, &tot_min);
  block_scan_i64(sum_w, sm, &tot_w);
  block_scan_i64(bad, sm, &tot_bad);
  if (t == 0) {
    io.meta[p * 4 + 0] = tot_min;
    io.meta[p * 4 + 1] = tot_w;
    io.meta[p * 4 + 2] = tot_bad;
  }
}

// Phase B for problem p (after phase A's global writes are visible).  lds: scratch of
// lds_bytes (>= 8 KiB); when the problem's segments fit they are staged there once.
__device__ inline void alloc_phase_b(const AllocIO& io, int p, char* lds, int lds_bytes) {
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int64_t hbase = (int64_t)p * NH;
  const int64_t nseg = (int64_t)NH * Gp;
  long long* sm = reinterpret_cast<long long*>(lds);                          // 4 slots
  unsigned long long* sel = reinterpret_cast<unsigned long long*>(lds + 64);  // prefix, rem, and, or
  unsigned long long* hist = reinterpret_cast<unsigned long long*>(lds + 128);  // 256 bins
  const unsigned long long* skey = io.seg_key + hbase * Gp;
  const unsigned* sw = io.seg_w + hbase * Gp;

  const long long tot_min = io.meta[p * 4 + 0], tot_w = io.meta[p * 4 + 1], tot_bad = io.meta[p * 4 + 2];
  const long long R = io.B[p] - tot_min;
  const bool infeasible = tot_bad != 0 || R < 0 || R > tot_w;
  const bool active = !infeasible && R > 0;

  // stage the segments in LDS when they fit (every later pass re-reads them)
  const int64_t cap = (lds_bytes - 4096) / 12;
  __syncthreads();
  if (nseg <= cap) {
    unsigned long long* lk = reinterpret_cast<unsigned long long*>(lds + 4096);
    unsigned* lw = reinterpret_cast<unsigned*>(lds + 4096 + nseg * 8);
    for (int64_t i = t; i < nseg; i += 256) { lk[i] = skey[i]; lw[i] = sw[i]; }
    skey = lk;
    sw = lw;
  }
  if (t == 0) { sel[0] = 0ull; sel[1] = (unsigned long long)R; sel[2] = ~0ull; sel[3] = 0ull; }
  __syncthreads();

  // weighted radix select of the threshold gain g*: W(> g*) < R <= W(>= g*)
  if (active) {
    // digits on which all live keys agree need no histogram
    unsigned long long k_and = ~0ull, k_or = 0ull;
    for (int64_t i = t; i < nseg; i += 256)
      if (sw[i]) { const unsigned long long key = skey[i]; k_and &= key; k_or |= key; }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      k_and &= ((unsigned long long)(unsigned)__shfl_xor((int)(k_and >> 32), o) << 32) | (unsigned)__shfl_xor((int)k_and, o);
      k_or |= ((unsigned long long)(unsigned)__shfl_xor((int)(k_or >> 32), o) << 32) | (unsigned)__shfl_xor((int)k_or, o);
    }
    if (lane == 0) { atomicAnd(&sel[2], k_and); atomicOr(&sel[3], k_or); }
    __syncthreads();
    const unsigned long long differ = sel[2] ^ sel[3];
    const unsigned long long common = sel[2];
    for (int shift = 56; shift >= 0; shift -= 8) {
      if (((differ >> shift) & 255ull) == 0ull) {
        // uniform: same digit for every live key, the wanted rank is unchanged
        __syncthreads();
        if (t == 0) sel[0] |= ((common >> shift) & 255ull) << shift;
        __syncthreads();
        continue;
      }
      hist[t] = 0ull;
      __syncthreads();
      const unsigned long long prefix = sel[0];
      for (int64_t i = t; i < nseg; i += 256) {
        const unsigned w = sw[i];
        if (w) {
          const unsigned long long key = skey[i];
          if (shift == 56 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
            atomicAdd(&hist[(key >> shift) & 255ull], (unsigned long long)w);
        }
      }
      __syncthreads();
      if (wave == 0) {
        // lane l owns the descending bins 4l .. 4l+3 (bin index 255-4l-k)
        long long v[4], s4 = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) { v[k] = (long long)hist[255 - 4 * lane - k]; s4 += v[k]; }
        long long incl = s4;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
          const long long up = shfl_up_i64(incl, o);
          if (lane >= o) incl += up;
        }
        long long before = incl - s4;
        const long long want = (long long)sel[1];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          if (before < want && want <= before + v[k]) {
            sel[0] = prefix | ((unsigned long long)(255 - 4 * lane - k) << shift);
            sel[1] = (unsigned long long)(want - before);
          }
          before += v[k];
        }
      }
      __syncthreads();
    }
  }
  const unsigned long long kstar = sel[0];
  const long long rem = active ? (long long)sel[1] : 0;

  // budgets: everything above g*, ties at g* in head order
  long long carry = 0;
  for (int h0 = 0; h0 < NH; h0 += 256) {
    const int h = h0 + t;
    long long gt = 0, eq = 0;
    if (h < NH && active) {
      for (int e = 0; e < Gp; ++e) {
        const unsigned w = sw[(int64_t)h * Gp + e];
        const unsigned long long key = skey[(int64_t)h * Gp + e];
        if (key > kstar) gt += w;
        else if (key == kstar) eq += w;
      }
    }
    long long tot;
    const long long eq_before = carry + block_scan_i64(eq, sm, &tot);
    carry += tot;
    if (h < NH) {
      long long take = rem - eq_before;
      take = take < 0 ? 0 : (take > eq ? eq : take);
      io.budgets[hbase + h] = (int32_t)(io.b_min[hbase + h] + gt + take);
    }
  }
  if (t == 0) io.status[p] = infeasible ? LUKV_ST_INFEASIBLE : 0;
}

}  // namespace lukv

#pragma clang fp contract(fast)
