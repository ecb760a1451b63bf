// Device code of step 2, the global head-level budget allocation (Sec. 4.2 "Efficient
// Optimization via Convex Hull Relaxation", Eq. 8-10; App. A.2 "Optimality of greedy
// allocation"), written so that it can run in its own kernel or as a few extra workgroups
// of other kernels of the path (it never looks at scores).
//
// The unit-by-unit greedy of the paper picks, B times, the head whose next unit has the
// largest marginal gain.  Gains are constant along a hull segment and strictly decreasing
// from one segment of a head to the next, so the greedy result is a weighted selection:
// find the gain g* at which the cumulated units (largest gain first) reach the remaining
// budget, give every head all its units above g*, and hand the units at exactly g* out in
// head order.
//   phase A: hull vertices by the chord criterion: knot g is a vertex of the upper concave hull
//            iff every chord from an earlier knot to g is strictly steeper than every chord
//            from g to a later knot (end knots always are).  All chords are independent fp64
//            divisions: no serial chain.  Two forms: one wave per (head, knot), for callers
//            that spread the knots over the prologues of another kernel's workgroups, and
//            sixteen threads per knot in workgroups of their own.
//   phase B: budgets.  Small problems (up to 1024 knots and 64 heads): 1024 threads, one per
//            knot; vertices are compacted into live segments, gains ranked in parallel, ties
//            handed out in head order.  Otherwise one workgroup per problem: a segment per
//            vertex (to the next vertex), clipped to (b_min, min(b_max, last knot)], gain as an
//            order-preserving 64-bit key; weighted radix select for g* (by the whole
//            workgroup, digits of up to 11 bits over the bits in which the keys differ, for
//            up to 1024 heads; a general form on one wave with 8-bit digits beyond that);
//            budgets per head, ties by a prefix sum over heads.  The row offsets (prefix sum
//            of all budgets) are written by whoever consumes the budgets next.
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
  int32_t* vertex;              // [n_problems * n_heads * n_grid] hull-vertex flags (phase A -> B)
  unsigned long long* seg_key;  // same shape; used when a problem's segments do not fit in LDS
  unsigned* seg_w;              // same
  int64_t B[LUKV_MAX_SEQS];
};

constexpr int kAllocPartsPerKnot = 16;  // threads sharing the chords of one knot in phase A

__host__ __device__ inline int alloc_blocks_a(int n_heads, int n_grid) {
  return (n_heads * n_grid * kAllocPartsPerKnot + 255) / 256;   // 256-thread blocks per problem
}

__device__ __forceinline__ unsigned long long gain_key(double x) {
  unsigned long long u = (unsigned long long)__double_as_longlong(x);
  if (x == 0.0) u = 0ull;  // -0 and +0 tie
  return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}

__device__ __forceinline__ long long shfl_up_i64(long long v, int o) {
  int lo = __shfl_up((int)(v & 0xFFFFFFFFll), o), hi = __shfl_up((int)(v >> 32), o);
  return ((long long)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ long long shfl_xor_i64(long long v, int o) {
  int lo = __shfl_xor((int)(v & 0xFFFFFFFFll), o), hi = __shfl_xor((int)(v >> 32), o);
  return ((long long)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ long long shfl_i64(long long v, int src) {
  int lo = __shfl((int)(v & 0xFFFFFFFFll), src), hi = __shfl((int)(v >> 32), src);
  return ((long long)hi << 32) | (unsigned)lo;
}

__device__ __forceinline__ double shfl_xor_f64(double v, int o) {
  const long long b = __double_as_longlong(v);
  const int lo = __shfl_xor((int)(b & 0xFFFFFFFFll), o), hi = __shfl_xor((int)(b >> 32), o);
  return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}

// Exclusive scan of one int64 per thread over the workgroup (<= 16 waves); sm has 16 slots.
__device__ __forceinline__ long long block_scan_i64(long long v, long long* sm, long long* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
  long long incl = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const long long up = shfl_up_i64(incl, o);
    if (lane >= o) incl += up;
  }
  __syncthreads();
  if (lane == 63) sm[wave] = incl;
  __syncthreads();
  long long before = 0, tot = 0;
  for (int w = 0; w < n_waves; ++w) {
    if (w < wave) before += sm[w];
    tot += sm[w];
  }
  *total = tot;
  return before + incl - v;
}

// Phase A: 256-thread block `blk` (0 .. alloc_blocks_a-1) of problem p.
__device__ inline void alloc_phase_a(const AllocIO& io, int p, int blk) {
  const int NH = io.n_heads, Gp = io.n_grid;
  const int unit = blk * 256 + threadIdx.x;
  const int item = unit / kAllocPartsPerKnot, part = unit % kAllocPartsPerKnot;
  const bool live = item < NH * Gp;
  const int h = live ? item / Gp : 0, g = live ? item - h * Gp : 0;
  const int64_t base = ((int64_t)p * NH + h) * Gp;
  const int32_t* n = io.knots + base;
  const float* U = io.curves + base;
  const int n_me = n[g];
  const double u_me = (double)U[g];
  double steep_in = INFINITY, steep_out = -INFINITY;
  if (live && g > 0 && g < Gp - 1) {
    // independent divisions, unrolled so that several are in flight
#pragma unroll 4
    for (int a = part; a < g; a += kAllocPartsPerKnot) {
      const double s = (u_me - (double)U[a]) / (double)(n_me - n[a]);
      steep_in = s < steep_in ? s : steep_in;
    }
#pragma unroll 4
    for (int c = g + 1 + part; c < Gp; c += kAllocPartsPerKnot) {
      const double s = ((double)U[c] - u_me) / (double)(n[c] - n_me);
      steep_out = s > steep_out ? s : steep_out;
    }
  }
#pragma unroll
  for (int o = 1; o < kAllocPartsPerKnot; o <<= 1) {
    const double i2 = shfl_xor_f64(steep_in, o), o2 = shfl_xor_f64(steep_out, o);
    steep_in = i2 < steep_in ? i2 : steep_in;
    steep_out = o2 > steep_out ? o2 : steep_out;
  }
  if (live && part == 0) io.vertex[base + g] = (g == 0 || g == Gp - 1) ? 1 : (steep_in > steep_out ? 1 : 0);
}

// Phase A for one knot by one wave, in two steps so that the loads can be issued before a
// workgroup's other loads and consumed after them: all 64 lanes call both with the same `item`
// (flat knot index over problems, heads and grid points); lane l takes the chord to knot l
// (grids of more than 64 points: the remaining chords are loaded in the second step).
struct AllocKnotLoad { float u_x, u_me; int32_t n_x, n_me; };

__device__ __forceinline__ AllocKnotLoad alloc_knot_load(const AllocIO& io, int64_t item) {
  const int Gp = io.n_grid, lane = threadIdx.x & 63;
  const int64_t hb = item / Gp * Gp;
  const int g = (int)(item - hb), x = lane < Gp ? lane : g;
  AllocKnotLoad ld;
  ld.u_x = io.curves[hb + x];
  ld.n_x = io.knots[hb + x];
  ld.u_me = io.curves[hb + g];
  ld.n_me = io.knots[hb + g];
  return ld;
}

__device__ __forceinline__ void alloc_knot_finish(const AllocIO& io, int64_t item, const AllocKnotLoad& ld) {
  const int Gp = io.n_grid, lane = threadIdx.x & 63;
  const int64_t hb = item / Gp * Gp;
  const int g = (int)(item - hb);
  const double u_me = (double)ld.u_me;
  const int n_me = ld.n_me;
  double steep_in = INFINITY, steep_out = -INFINITY;
  if (lane < g) {
    steep_in = (u_me - (double)ld.u_x) / (double)(n_me - ld.n_x);
  } else if (lane > g && lane < Gp) {
    steep_out = ((double)ld.u_x - u_me) / (double)(ld.n_x - n_me);
  }
  for (int x = lane + 64; x < Gp; x += 64) {
    if (x < g) {
      const double s = (u_me - (double)io.curves[hb + x]) / (double)(n_me - io.knots[hb + x]);
      steep_in = s < steep_in ? s : steep_in;
    } else if (x > g) {
      const double s = ((double)io.curves[hb + x] - u_me) / (double)(io.knots[hb + x] - n_me);
      steep_out = s > steep_out ? s : steep_out;
    }
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const double i2 = shfl_xor_f64(steep_in, o), o2 = shfl_xor_f64(steep_out, o);
    steep_in = i2 < steep_in ? i2 : steep_in;
    steep_out = o2 > steep_out ? o2 : steep_out;
  }
  if (lane == 0) io.vertex[item] = (g == 0 || g == Gp - 1) ? 1 : (steep_in > steep_out ? 1 : 0);
}

// Knots per scoring workgroup when phase A is spread over the prologues of n_wgs workgroups of
// four waves (one knot per wave at most); 0 when the problem is too large for that.
__host__ __device__ inline int alloc_spread_knots(int64_t n_knots, int64_t n_wgs) {
  if (n_wgs <= 0) return 0;
  const int64_t kp = (n_knots + n_wgs - 1) / n_wgs;
  return kp <= 4 ? (int)kp : 0;
}

// Phase B, general form, for problem p (after phase A's flags are visible): any number of heads
// and segments, any workgroup size that is a multiple of 64 from 256 to 1024; lds: scratch of
// lds_bytes (>= 32 KiB), free for this call.  Used when alloc_phase_b_mid below does not apply.
// Everything a thread walks more than once (vertex flags, knots, curves, segments, per-head
// sums) is staged in LDS when the problem fits (up to 1024 segments and 1024 heads; larger
// problems use the workspace and global memory, slower but the same arithmetic).  The radix
// select itself is wave-synchronous on wave 0, its segments held in registers, so a small
// problem pays no workgroup barrier per digit.
__device__ inline void alloc_phase_b_generic(const AllocIO& io, int p, char* lds, int lds_bytes) {
  constexpr int kRegSegs = 16;              // segments per lane that wave 0 keeps in registers
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x, nt = blockDim.x;
  const int lane = t & 63, wave = t >> 6;
  const int64_t hbase = (int64_t)p * NH;
  const int64_t nseg = (int64_t)NH * Gp;
  long long* sm = reinterpret_cast<long long*>(lds);                            // 16 slots
  long long* red = reinterpret_cast<long long*>(lds + 128);                     // sum b_min, sum w, bad
  unsigned long long* sel = reinterpret_cast<unsigned long long*>(lds + 160);   // g*, ties, and, or
  unsigned long long* hist = reinterpret_cast<unsigned long long*>(lds + 192);  // 256 bins of units
  unsigned* hcnt = reinterpret_cast<unsigned*>(lds + 192 + 2048);               // 256 bins of segments
  const int32_t* vtx = io.vertex + hbase * Gp;
  const int32_t* kn = io.knots + hbase * Gp;
  const float* cu = io.curves + hbase * Gp;

  // LDS plan (small problems, <= 1024 segments and <= 64 heads): vertex bit masks, per-head
  // bounds and sums, knots, curves and the segments themselves all live in LDS
  const int words = (Gp + 63) / 64;                      // mask words per head
  const bool small = nseg <= 1024 && NH <= 64 && NH * words <= 96 && lds_bytes >= 32768;
  unsigned long long* l_mask = reinterpret_cast<unsigned long long*>(lds + 3328);   // [NH][words]
  int32_t* l_lb = reinterpret_cast<int32_t*>(lds + 4096);                           // b_min per head
  int32_t* l_cp = l_lb + 64;                                                        // cap per head
  long long* h_gt = reinterpret_cast<long long*>(lds + 4608);                       // per-head sums
  long long* h_eq = h_gt + 64;
  int32_t* l_kn = reinterpret_cast<int32_t*>(lds + 5632);
  float* l_cu = reinterpret_cast<float*>(lds + 5632 + nseg * 4);
  unsigned* l_w = reinterpret_cast<unsigned*>(lds + 5632 + nseg * 8);
  unsigned long long* l_key = reinterpret_cast<unsigned long long*>(lds + 5632 + (nseg * 12 + 7) / 8 * 8);
  unsigned long long* skey = small ? l_key : io.seg_key + hbase * Gp;
  unsigned* sw = small ? l_w : io.seg_w + hbase * Gp;
  __syncthreads();
  if (t == 0) {
    red[0] = red[1] = red[2] = 0;
    sel[0] = 0ull; sel[1] = 0ull; sel[2] = ~0ull; sel[3] = 0ull;
  }
  if (small) {
    // every global load of the staging is issued before the first barrier
    for (int i = t; i < NH * words; i += nt) l_mask[i] = 0ull;
    for (int h = t; h < NH; h += nt) {
      l_lb[h] = io.b_min[hbase + h];
      const int32_t last = kn[(int64_t)h * Gp + Gp - 1], bm = io.b_max[hbase + h];
      l_cp[h] = bm < last ? bm : last;
      h_gt[h] = 0;
      h_eq[h] = 0;
    }
    if (nseg <= nt) {
      const bool in = t < (int)nseg;
      const int32_t vk = in ? kn[t] : 0;
      const float vc = in ? cu[t] : 0.f;
      const int32_t vv = in ? vtx[t] : 0;
      __syncthreads();
      if (in) {
        l_kn[t] = vk;
        l_cu[t] = vc;
        if (vv) { const int h = t / Gp, g = t - h * Gp; atomicOr(&l_mask[h * words + (g >> 6)], 1ull << (g & 63)); }
      }
    } else {
      __syncthreads();
      for (int i = t; i < (int)nseg; i += nt) {
        l_kn[i] = kn[i];
        l_cu[i] = cu[i];
        if (vtx[i]) { const int h = i / Gp, g = i - h * Gp; atomicOr(&l_mask[h * words + (g >> 6)], 1ull << (g & 63)); }
      }
    }
  }
  __syncthreads();

  // one segment per vertex (to the next vertex), clipped to (b_min, cap]
  long long sum_min = 0, sum_w = 0, bad = 0;
  unsigned long long k_and = ~0ull, k_or = 0ull;
  for (int64_t i = t; i < nseg; i += nt) {
    const int h = (int)(i / Gp), g = (int)(i - (int64_t)h * Gp);
    const int64_t hb = (int64_t)h * Gp;
    const long long lb = small ? l_lb[h] : io.b_min[hbase + h];
    const long long cp = small ? l_cp[h] : min((long long)io.b_max[hbase + h], (long long)kn[hb + Gp - 1]);
    if (g == 0) {
      if (lb < 0 || lb > cp) bad = 1;
      sum_min += lb;
    }
    unsigned w = 0;
    unsigned long long key = 0;
    bool is_vertex;
    int c = g + 1;   // next vertex; the last knot is always one
    if (small) {
      const unsigned long long* mk = l_mask + h * words;
      is_vertex = (mk[g >> 6] >> (g & 63)) & 1ull;
      if (is_vertex && g < Gp - 1) {
        int wd = c >> 6;
        unsigned long long m = mk[wd] & (~0ull << (c & 63));
        while (m == 0ull && wd + 1 < words) m = mk[++wd];
        c = m ? wd * 64 + __ffsll((long long)m) - 1 : Gp - 1;
      }
    } else {
      is_vertex = vtx[i] != 0;
      if (is_vertex) while (c < Gp - 1 && !vtx[hb + c]) ++c;
    }
    if (g < Gp - 1 && is_vertex) {
      const long long na = small ? l_kn[i] : kn[i], nb = small ? l_kn[hb + c] : kn[hb + c];
      const double ua = (double)(small ? l_cu[i] : cu[i]), ub = (double)(small ? l_cu[hb + c] : cu[hb + c]);
      const long long lo = max(na, lb), hi = min(nb, cp);
      w = hi > lo ? (unsigned)(hi - lo) : 0u;
      key = gain_key((ub - ua) / (double)(nb - na));
    }
    skey[i] = key;
    sw[i] = w;
    sum_w += w;
    if (w) { k_and &= key; k_or |= key; }
  }
  // workgroup sums.  Small problems: the segments of a head tile (max(b_min, first knot), cap],
  // so the units on offer and the minimum retention are sums over heads, which wave 0 takes
  // from LDS; the waves that hold live segments only reduce the AND / OR of their keys (DPP
  // steps, 64-bit values as two halves), one LDS atomic per wave.
  if (small && nseg <= nt) {
    auto add = [](unsigned a, unsigned b) { return a + b; };
    auto band = [](unsigned a, unsigned b) { return a & b; };
    auto bor = [](unsigned a, unsigned b) { return a | b; };
    if (wave == 0) {
      const bool live = lane < NH;
      const long long lb = live ? l_lb[lane] : 0, cp = live ? l_cp[lane] : 0;
      const long long n0 = live ? l_kn[lane * Gp] : 0;
      const bool head_bad = live && (lb < 0 || lb > cp);
      const long long from = lb > n0 ? lb : n0;
      const unsigned offer = !head_bad && cp > from ? (unsigned)(cp - from) : 0u;   // < 2^31
      const unsigned keep = head_bad ? 0u : (unsigned)lb;
      // sums of 16-bit pieces cannot overflow a lane
      const unsigned m_lo = wave_reduce_to_last(keep & 0xFFFFu, 0u, add), m_hi = wave_reduce_to_last(keep >> 16, 0u, add);
      const unsigned w_lo = wave_reduce_to_last(offer & 0xFFFFu, 0u, add), w_hi = wave_reduce_to_last(offer >> 16, 0u, add);
      const unsigned long long any_bad = __ballot(head_bad);
      if (lane == 63) {
        red[0] = (long long)(((unsigned long long)m_hi << 16) + m_lo);
        red[1] = (long long)(((unsigned long long)w_hi << 16) + w_lo);
        red[2] = any_bad ? 1 : 0;
      }
    }
    if (__ballot(sum_w != 0) != 0ull) {
      const unsigned a_lo = wave_reduce_to_last((unsigned)k_and, ~0u, band);
      const unsigned a_hi = wave_reduce_to_last((unsigned)(k_and >> 32), ~0u, band);
      const unsigned o_lo = wave_reduce_to_last((unsigned)k_or, 0u, bor);
      const unsigned o_hi = wave_reduce_to_last((unsigned)(k_or >> 32), 0u, bor);
      if (lane == 63) {
        atomicAnd(&sel[2], ((unsigned long long)a_hi << 32) | a_lo);
        atomicOr(&sel[3], ((unsigned long long)o_hi << 32) | o_lo);
      }
    }
  } else {
    // most threads hold nothing, so only the others touch the LDS counters
    if (sum_min) atomicAdd(reinterpret_cast<unsigned long long*>(&red[0]), (unsigned long long)sum_min);
    if (sum_w) {
      atomicAdd(reinterpret_cast<unsigned long long*>(&red[1]), (unsigned long long)sum_w);
      atomicAnd(&sel[2], k_and);
      atomicOr(&sel[3], k_or);
    }
    if (bad) atomicAdd(reinterpret_cast<unsigned long long*>(&red[2]), 1ull);
  }
  __syncthreads();
  const long long R = io.B[p] - red[0];
  const bool infeasible = red[2] != 0 || R < 0 || R > red[1];
  const bool active = !infeasible && R > 0;

  // weighted radix select of the threshold gain g*: W(> g*) < R <= W(>= g*)
  // fast form: one segment per thread, 32-bit unit counts, digits of up to 11 bits over the
  // bits in which the live keys differ, from the top varying bit down; stops as soon as the
  // chosen bin holds a single segment
  const bool fast = small && nt == 1024 && lds_bytes >= 49152 && red[1] < (1ll << 31);
  if (active && fast) {
    unsigned* bh = reinterpret_cast<unsigned*>(lds + 32768);   // kHistBins unit counts
    unsigned* bc = bh + kHistBins;                             // kHistBins segment counts
    unsigned* spart = reinterpret_cast<unsigned*>(sm);         // 16 slots for the scans
    unsigned* pick32 = reinterpret_cast<unsigned*>(lds + 152); // bin, units still wanted
    const unsigned long long differ = sel[2] ^ sel[3];
    const unsigned long long mykey = t < nseg ? skey[t] : 0ull;
    const unsigned myw = t < nseg ? sw[t] : 0u;
    int rest = differ ? 64 - __clzll((long long)differ) : 0;     // low bits still open
    unsigned long long prefix = rest == 64 ? 0ull : sel[2] & ~((1ull << rest) - 1ull);
    unsigned want = (unsigned)R;
    bool single = false;
    while (rest > 0) {
      const int sh = rest > 11 ? rest - 11 : 0;
      const unsigned mask = (1u << (rest - sh)) - 1u;
      const unsigned long long hi_mask = rest == 64 ? 0ull : ~((1ull << rest) - 1ull);
      __syncthreads();
      bh[t] = 0u; bh[t + 1024] = 0u;
      bc[t] = 0u; bc[t + 1024] = 0u;
      __syncthreads();
      const bool in = myw != 0u && (mykey & hi_mask) == (prefix & hi_mask);
      const unsigned d = (unsigned)(mykey >> sh) & mask;
      if (in) { atomicAdd(&bh[d], myw); atomicAdd(&bc[d], 1u); }
      __syncthreads();
      const unsigned a1 = bh[2047 - 2 * t], a0 = bh[2046 - 2 * t];
      const unsigned before = block_scan_u32(a1 + a0, spart);
      if (before < want && want <= before + a1) { pick32[0] = 2047 - 2 * t; pick32[1] = want - before; }
      else if (before + a1 < want && want <= before + a1 + a0) { pick32[0] = 2046 - 2 * t; pick32[1] = want - before - a1; }
      __syncthreads();
      const unsigned bin = pick32[0];
      want = pick32[1];
      prefix |= (unsigned long long)bin << sh;
      rest = sh;
      if (bc[bin] == 1u) {
        // a single segment is left in the chosen bin: its key is g*
        if (in && d == bin) sel[0] = mykey;
        single = true;
        break;
      }
    }
    if (!single && t == 0) sel[0] = prefix;
    if (t == 0) sel[1] = (unsigned long long)want;
  } else if (active && wave == 0) {
    const unsigned long long differ = sel[2] ^ sel[3], common = sel[2];
    const bool in_regs = nseg <= 64 * kRegSegs;
    unsigned long long rkey[kRegSegs];
    unsigned rw[kRegSegs];
    if (in_regs) {
#pragma unroll
      for (int u = 0; u < kRegSegs; ++u) {
        const int64_t i = lane + 64 * u;
        rw[u] = i < nseg ? sw[i] : 0u;
        rkey[u] = i < nseg ? skey[i] : 0ull;
      }
    }
    unsigned long long prefix = 0ull;
    long long want = R;
    for (int shift = 56; shift >= 0; shift -= 8) {
      if (((differ >> shift) & 255ull) == 0ull) {
        prefix |= ((common >> shift) & 255ull) << shift;   // every live key has this digit
        continue;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) { hist[4 * lane + k] = 0ull; hcnt[4 * lane + k] = 0u; }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      if (in_regs) {
#pragma unroll
        for (int u = 0; u < kRegSegs; ++u)
          if (rw[u] && (shift == 56 || (rkey[u] >> (shift + 8)) == (prefix >> (shift + 8)))) {
            atomicAdd(&hist[(rkey[u] >> shift) & 255ull], (unsigned long long)rw[u]);
            atomicAdd(&hcnt[(rkey[u] >> shift) & 255ull], 1u);
          }
      } else {
        for (int64_t i = lane; i < nseg; i += 64) {
          const unsigned w = sw[i];
          if (w) {
            const unsigned long long key = skey[i];
            if (shift == 56 || (key >> (shift + 8)) == (prefix >> (shift + 8)))
              atomicAdd(&hist[(key >> shift) & 255ull], (unsigned long long)w);
          }
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
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
      int found_bin = -1;
      long long found_rem = 0;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        if (before < want && want <= before + v[k]) { found_bin = 255 - 4 * lane - k; found_rem = want - before; }
        before += v[k];
      }
      const unsigned long long who = __ballot(found_bin >= 0);   // exactly one lane
      const int src = __ffsll((long long)who) - 1;
      const int bin = __shfl(found_bin, src);
      want = shfl_i64(found_rem, src);
      prefix |= (unsigned long long)bin << shift;
      if (in_regs && hcnt[bin] == 1u) {
        // a single segment is left in the chosen bin: its key is g*, no further digits needed
        unsigned long long mine = 0ull;
#pragma unroll
        for (int u = 0; u < kRegSegs; ++u)
          if (rw[u] && (rkey[u] >> shift) == (prefix >> shift)) mine = rkey[u];
        const unsigned long long owner = __ballot(mine != 0ull);
        prefix = (unsigned long long)shfl_i64((long long)mine, __ffsll((long long)owner) - 1);
        break;
      }
      __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
    if (lane == 0) { sel[0] = prefix; sel[1] = (unsigned long long)want; }
  }
  __syncthreads();
  const unsigned long long kstar = sel[0];
  const long long rem = active ? (long long)sel[1] : 0;

  // budgets: everything above g*, ties at g* in head order
  const bool head_lds = small;
  if (head_lds) {
    if (active) {
      for (int i = t; i < (int)nseg; i += nt) {
        const unsigned w = sw[i];
        if (w) {
          const unsigned long long key = skey[i];
          if (key > kstar) atomicAdd(reinterpret_cast<unsigned long long*>(&h_gt[i / Gp]), (unsigned long long)w);
          else if (key == kstar) atomicAdd(reinterpret_cast<unsigned long long*>(&h_eq[i / Gp]), (unsigned long long)w);
        }
      }
    }
    __syncthreads();
  }
  if (fast) {
    // at most 64 heads, sums below 2^31: wave 0 alone, ties in head order by a wave scan
    if (wave == 0) {
      const bool live = lane < NH;
      const unsigned gt = live && active ? (unsigned)h_gt[live ? lane : 0] : 0u;
      const unsigned eq = live && active ? (unsigned)h_eq[live ? lane : 0] : 0u;
      const long long eq_before = (long long)(wave_scan_incl(eq) - eq);
      if (live) {
        long long take = rem - eq_before;
        take = take < 0 ? 0 : (take > (long long)eq ? (long long)eq : take);
        io.budgets[hbase + lane] = (int32_t)(l_lb[lane] + (long long)gt + take);
      }
    }
    if (t == 0) io.status[p] = infeasible ? LUKV_ST_INFEASIBLE : 0;
    return;
  }
  long long carry = 0;
  for (int h0 = 0; h0 < NH; h0 += nt) {
    const int h = h0 + t;
    long long gt = 0, eq = 0;
    if (h < NH && active) {
      if (head_lds) {
        gt = h_gt[h];
        eq = h_eq[h];
      } else {
        for (int e = 0; e < Gp; ++e) {
          const unsigned w = sw[(int64_t)h * Gp + e];
          const unsigned long long key = skey[(int64_t)h * Gp + e];
          if (key > kstar) gt += w;
          else if (key == kstar) eq += w;
        }
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

constexpr int kAllocLdsBytes = 61696;   // LDS the 1024-thread form of phase B needs

// Weighted radix select of the threshold key over the problem's segments (key, units), by the
// whole workgroup of 1024 threads: digits of up to 11 bits over the bits in which the live keys
// differ (and_keys / or_keys), from the top varying bit down; `want` units are wanted counting
// from the largest key; stops as soon as the chosen bin holds a single segment.  W is the type
// that holds unit counts (unsigned when the total fits 31 bits).  Returns (g*, units wanted at
// g*) through out[0], out[1]; every thread calls it.
template <class W, class KeyPtr, class WPtr>
__device__ __forceinline__ void alloc_block_select(KeyPtr skey, WPtr sw, int nseg, unsigned long long and_keys,
                                                   unsigned long long or_keys, W want, W* bh, unsigned* bc,
                                                   void* scan_scratch, W* pick, unsigned long long* out) {
  const int t = threadIdx.x;
  const unsigned long long differ = and_keys ^ or_keys;
  int rest = differ ? 64 - __clzll((long long)differ) : 0;     // low bits still open
  unsigned long long prefix = rest == 64 ? 0ull : and_keys & ~((1ull << rest) - 1ull);
  bool single = false;
  while (rest > 0) {
    const int sh = rest > 11 ? rest - 11 : 0;
    const unsigned mask = (1u << (rest - sh)) - 1u;
    const unsigned long long hi_mask = rest == 64 ? 0ull : ~((1ull << rest) - 1ull);
    __syncthreads();
    bh[t] = 0; bh[t + 1024] = 0;
    bc[t] = 0u; bc[t + 1024] = 0u;
    __syncthreads();
    for (int i = t; i < nseg; i += 1024) {
      const unsigned w = sw[i];
      if (w) {
        const unsigned long long key = skey[i];
        if ((key & hi_mask) == (prefix & hi_mask)) {
          const unsigned d = (unsigned)(key >> sh) & mask;
          atomicAdd(&bh[d], (W)w);
          atomicAdd(&bc[d], 1u);
        }
      }
    }
    __syncthreads();
    const W a1 = bh[2047 - 2 * t], a0 = bh[2046 - 2 * t];
    W before;
    if constexpr (sizeof(W) == 4) {
      before = block_scan_u32(a1 + a0, reinterpret_cast<unsigned*>(scan_scratch));
    } else {
      long long tot;
      before = (W)block_scan_i64((long long)(a1 + a0), reinterpret_cast<long long*>(scan_scratch), &tot);
    }
    if (before < want && want <= before + a1) { pick[0] = (W)(2047 - 2 * t); pick[1] = want - before; }
    else if (before + a1 < want && want <= before + a1 + a0) { pick[0] = (W)(2046 - 2 * t); pick[1] = want - before - a1; }
    __syncthreads();
    const unsigned bin = (unsigned)pick[0];
    want = pick[1];
    prefix |= (unsigned long long)bin << sh;
    rest = sh;
    if (bc[bin] == 1u) {
      // a single segment is left in the chosen bin: its key is g*
      for (int i = t; i < nseg; i += 1024) {
        const unsigned long long key = skey[i];
        if (sw[i] && (key >> sh) == (prefix >> sh)) out[0] = key;
      }
      single = true;
      break;
    }
  }
  if (!single && t == 0) out[0] = prefix;
  if (t == 0) out[1] = (unsigned long long)want;
}

// Phase B for problems of up to 1024 heads (and 1024 mask words), by a workgroup of 1024
// threads with kAllocLdsBytes of LDS: vertex flags as bit masks and per-head bounds in LDS;
// knots, curves and segments too when there are at most 1024 segments, else read from global
// memory / kept in the workspace; block-wide select; per-head sums by a few threads per head.
__device__ inline void alloc_phase_b_mid(const AllocIO& io, int p, char* lds) {
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int64_t hbase = (int64_t)p * NH;
  const int nseg = NH * Gp;
  const int words = (Gp + 63) / 64;
  unsigned* spart = reinterpret_cast<unsigned*>(lds);                              // scan scratch (128 B)
  long long* red = reinterpret_cast<long long*>(lds + 128);                        // sum b_min, units on offer, bad
  unsigned long long* sel = reinterpret_cast<unsigned long long*>(lds + 160);      // g*, ties, and, or
  unsigned long long* pick = reinterpret_cast<unsigned long long*>(lds + 192);     // bin, units still wanted
  unsigned long long* l_mask = reinterpret_cast<unsigned long long*>(lds + 256);   // [NH][words] <= 1024
  int32_t* l_lb = reinterpret_cast<int32_t*>(lds + 8448);                          // b_min per head
  int32_t* l_cp = reinterpret_cast<int32_t*>(lds + 12544);                         // cap per head
  int32_t* l_kn = reinterpret_cast<int32_t*>(lds + 16640);                         // <= 1024 segments:
  float* l_cu = reinterpret_cast<float*>(lds + 20736);                             //   knots, curves,
  unsigned* l_w = reinterpret_cast<unsigned*>(lds + 24832);                        //   units and keys
  unsigned long long* l_key = reinterpret_cast<unsigned long long*>(lds + 28928);
  char* big = lds + 37120;                                                         // 24 KiB: select, then sums
  long long* h_gt = reinterpret_cast<long long*>(big);                             // per-head sums
  long long* h_eq = h_gt + 1024;
  const int32_t* vtx = io.vertex + hbase * Gp;
  const int32_t* kn = io.knots + hbase * Gp;
  const float* cu = io.curves + hbase * Gp;
  const bool in_lds = nseg <= 1024;
  auto add = [](unsigned a, unsigned b) { return a + b; };
  auto band = [](unsigned a, unsigned b) { return a & b; };
  auto bor = [](unsigned a, unsigned b) { return a | b; };

  __syncthreads();
  if (t == 0) {
    red[0] = red[1] = red[2] = 0;
    sel[0] = 0ull; sel[1] = 0ull; sel[2] = ~0ull; sel[3] = 0ull;
  }
  for (int i = t; i < NH * words; i += 1024) l_mask[i] = 0ull;
  // staging: every global load is issued before the first barrier
  const bool head = t < NH;
  const long long lb = head ? io.b_min[hbase + t] : 0;
  const long long n0 = head ? kn[(int64_t)t * Gp] : 0, n_last = head ? kn[(int64_t)t * Gp + Gp - 1] : 0;
  const long long bm = head ? io.b_max[hbase + t] : 0;
  const bool mine = in_lds && t < nseg;
  const int32_t vk = mine ? kn[t] : 0;
  const float vc = mine ? cu[t] : 0.f;
  const int32_t vv = mine ? vtx[t] : 0;
  __syncthreads();
  const long long cp = bm < n_last ? bm : n_last;
  if (head) { l_lb[t] = (int32_t)lb; l_cp[t] = (int32_t)cp; }
  if (in_lds) {
    if (mine) {
      l_kn[t] = vk;
      l_cu[t] = vc;
      if (vv) { const int h = t / Gp, g = t - h * Gp; atomicOr(&l_mask[h * words + (g >> 6)], 1ull << (g & 63)); }
    }
  } else {
    for (int i = t; i < nseg; i += 1024)
      if (vtx[i]) { const int h = i / Gp, g = i - h * Gp; atomicOr(&l_mask[h * words + (g >> 6)], 1ull << (g & 63)); }
  }
  // The segments of a head tile (max(b_min, first knot), cap], so the units on offer and the
  // minimum retention are sums over heads: wave reductions on 16-bit pieces (a lane cannot
  // overflow), one LDS atomic per wave.
  if (wave * 64 < NH) {
    const bool head_bad = head && (lb < 0 || lb > cp);
    const long long from = lb > n0 ? lb : n0;
    const unsigned offer = head && !head_bad && cp > from ? (unsigned)(cp - from) : 0u;   // < 2^31
    const unsigned keep = head && !head_bad ? (unsigned)lb : 0u;
    const unsigned m_lo = wave_reduce_to_last(keep & 0xFFFFu, 0u, add), m_hi = wave_reduce_to_last(keep >> 16, 0u, add);
    const unsigned w_lo = wave_reduce_to_last(offer & 0xFFFFu, 0u, add), w_hi = wave_reduce_to_last(offer >> 16, 0u, add);
    const unsigned long long any_bad = __ballot(head_bad);
    if (lane == 63) {
      atomicAdd(reinterpret_cast<unsigned long long*>(&red[0]), ((unsigned long long)m_hi << 16) + m_lo);
      atomicAdd(reinterpret_cast<unsigned long long*>(&red[1]), ((unsigned long long)w_hi << 16) + w_lo);
      if (any_bad) atomicAdd(reinterpret_cast<unsigned long long*>(&red[2]), 1ull);
    }
  }
  __syncthreads();

  // one segment per vertex (to the next vertex), clipped to (b_min, cap]
  unsigned long long* skey = in_lds ? l_key : io.seg_key + hbase * Gp;
  unsigned* sw = in_lds ? l_w : io.seg_w + hbase * Gp;
  unsigned long long k_and = ~0ull, k_or = 0ull;
  bool any_w = false;
  for (int i = t; i < nseg; i += 1024) {
    const int h = i / Gp, g = i - h * Gp;
    const int hb = h * Gp;
    const unsigned long long* mk = l_mask + h * words;
    unsigned w = 0;
    unsigned long long key = 0;
    if (g < Gp - 1 && ((mk[g >> 6] >> (g & 63)) & 1ull)) {
      int c = g + 1, wd = c >> 6;            // next vertex; the last knot is always one
      unsigned long long m = mk[wd] & (~0ull << (c & 63));
      while (m == 0ull && wd + 1 < words) m = mk[++wd];
      c = m ? wd * 64 + __ffsll((long long)m) - 1 : Gp - 1;
      const long long na = in_lds ? l_kn[i] : kn[i], nb = in_lds ? l_kn[hb + c] : kn[hb + c];
      const double ua = (double)(in_lds ? l_cu[i] : cu[i]), ub = (double)(in_lds ? l_cu[hb + c] : cu[hb + c]);
      const long long hlb = l_lb[h], hcp = l_cp[h];
      const long long lo = max(na, hlb), hi = min(nb, hcp);
      w = hi > lo ? (unsigned)(hi - lo) : 0u;
      key = gain_key((ub - ua) / (double)(nb - na));
    }
    skey[i] = key;
    sw[i] = w;
    if (w) { k_and &= key; k_or |= key; any_w = true; }
  }
  if (__ballot(any_w) != 0ull) {
    const unsigned a_lo = wave_reduce_to_last((unsigned)k_and, ~0u, band);
    const unsigned a_hi = wave_reduce_to_last((unsigned)(k_and >> 32), ~0u, band);
    const unsigned o_lo = wave_reduce_to_last((unsigned)k_or, 0u, bor);
    const unsigned o_hi = wave_reduce_to_last((unsigned)(k_or >> 32), 0u, bor);
    if (lane == 63) {
      atomicAnd(&sel[2], ((unsigned long long)a_hi << 32) | a_lo);
      atomicOr(&sel[3], ((unsigned long long)o_hi << 32) | o_lo);
    }
  }
  __syncthreads();
  const long long R = io.B[p] - red[0];
  const bool infeasible = red[2] != 0 || R < 0 || R > red[1];
  const bool active = !infeasible && R > 0;
  const bool narrow = red[1] < (1ll << 31);     // unit counts fit 32 bits

  // threshold gain g*: W(> g*) < R <= W(>= g*)
  if (active) {
    if (narrow)
      alloc_block_select<unsigned>(skey, sw, nseg, sel[2], sel[3], (unsigned)R, reinterpret_cast<unsigned*>(big),
                                   reinterpret_cast<unsigned*>(big + 16384), spart, reinterpret_cast<unsigned*>(pick), sel);
    else
      alloc_block_select<unsigned long long>(skey, sw, nseg, sel[2], sel[3], (unsigned long long)R,
                                             reinterpret_cast<unsigned long long*>(big),
                                             reinterpret_cast<unsigned*>(big + 16384), spart, pick, sel);
  }
  __syncthreads();
  const unsigned long long kstar = sel[0];
  const long long rem = active ? (long long)sel[1] : 0;

  // budgets: everything above g*, ties at g* in head order.  A power-of-two number of threads
  // per head sums that head's segments; the parts meet in LDS.
  for (int h = t; h < NH; h += 1024) { h_gt[h] = 0; h_eq[h] = 0; }
  __syncthreads();
  if (active) {
    int parts = 1;
    while (parts < 64 && parts * 2 * NH <= 1024) parts *= 2;
    const int h = t / parts, part = t - h * parts;
    if (h < NH) {
      long long gt = 0, eq = 0;
      for (int e = part; e < Gp; e += parts) {
        const unsigned w = sw[h * Gp + e];
        if (w) {
          const unsigned long long key = skey[h * Gp + e];
          if (key > kstar) gt += w;
          else if (key == kstar) eq += w;
        }
      }
      if (gt) atomicAdd(reinterpret_cast<unsigned long long*>(&h_gt[h]), (unsigned long long)gt);
      if (eq) atomicAdd(reinterpret_cast<unsigned long long*>(&h_eq[h]), (unsigned long long)eq);
    }
  }
  __syncthreads();
  {
    const long long gt = head ? h_gt[t] : 0, eq = head ? h_eq[t] : 0;
    long long eq_before;
    if (narrow) {
      eq_before = (long long)block_scan_u32((unsigned)eq, spart);
    } else {
      long long tot;
      eq_before = block_scan_i64(eq, reinterpret_cast<long long*>(spart), &tot);
    }
    if (head) {
      long long take = rem - eq_before;
      take = take < 0 ? 0 : (take > eq ? eq : take);
      io.budgets[hbase + t] = (int32_t)(lb + gt + take);
    }
  }
  if (t == 0) io.status[p] = infeasible ? LUKV_ST_INFEASIBLE : 0;
}

// Phase B for a small problem (at most 1024 knots and 64 heads) by a workgroup of 1024 threads
// with 32 KiB of LDS: one thread per knot; the hull segments that still offer units are compacted
// into a list, and the threshold gain is found by ranking every such segment against all others
// (a few hundred at most), which needs no digit passes.  Same result as the other forms.
// What a thread of alloc_phase_b_small reads from global memory, so that a caller can issue the
// loads early (they are cold: nothing else touches the curves) and run the phase later.
struct AllocSmallLoad { int32_t vk, vv; float vc; int32_t lb, bm, n0, n_last; };

__device__ __forceinline__ AllocSmallLoad alloc_small_load(const AllocIO& io, int p) {
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x;
  const int64_t hbase = (int64_t)p * NH;
  const bool mine = t < NH * Gp, head = t < NH;
  const int32_t* kn = io.knots + hbase * Gp;
  AllocSmallLoad ld;
  ld.vk = mine ? kn[t] : 0;
  ld.vc = mine ? io.curves[hbase * Gp + t] : 0.f;
  ld.vv = mine ? io.vertex[hbase * Gp + t] : 0;
  ld.lb = head ? io.b_min[hbase + t] : 0;
  ld.bm = head ? io.b_max[hbase + t] : 0;
  ld.n0 = head ? kn[(int64_t)t * Gp] : 0;
  ld.n_last = head ? kn[(int64_t)t * Gp + Gp - 1] : 0;
  return ld;
}

// budgets_lds (may be NULL): LDS array of n_heads budgets for the caller's own use;
// write_out: whether this workgroup writes budgets and status to global memory (several
// workgroups may run the same problem redundantly).
__device__ inline void alloc_phase_b_small(const AllocIO& io, int p, char* lds, const AllocSmallLoad& pre,
                                           int32_t* budgets_lds, bool write_out) {
  const int NH = io.n_heads, Gp = io.n_grid, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int64_t hbase = (int64_t)p * NH;
  const int nseg = NH * Gp;
  const int words = (Gp + 63) / 64;                       // NH * words <= 80
  unsigned long long* l_mask = reinterpret_cast<unsigned long long*>(lds);           // [NH][words] <= 128
  long long* red = reinterpret_cast<long long*>(lds + 1024);                         // sum b_min, units on offer, bad
  unsigned long long* sel = reinterpret_cast<unsigned long long*>(lds + 1056);       // g*, units wanted at g*
  unsigned* n_live = reinterpret_cast<unsigned*>(lds + 1072);
  int32_t* l_lb = reinterpret_cast<int32_t*>(lds + 1088);                            // [64]
  int32_t* l_cp = l_lb + 64;                                                         // [64]
  unsigned long long* h_gt = reinterpret_cast<unsigned long long*>(lds + 1600);      // [64]
  unsigned long long* h_eq = h_gt + 64;                                              // [64]
  int32_t* l_kn = reinterpret_cast<int32_t*>(lds + 2624);                            // [1024]
  float* l_cu = reinterpret_cast<float*>(lds + 6720);                                // [1024]
  unsigned long long* live_key = reinterpret_cast<unsigned long long*>(lds + 10816); // [1024]
  unsigned* live_w = reinterpret_cast<unsigned*>(lds + 19008);                       // [1024]
  unsigned short* live_h = reinterpret_cast<unsigned short*>(lds + 23104);           // [1024] -> 25152
  auto add = [](unsigned a, unsigned b) { return a + b; };
  __syncthreads();
  const bool mine = t < nseg, head = t < NH;
  const int32_t vk = pre.vk, vv = pre.vv;
  const float vc = pre.vc;
  const long long lb = pre.lb, bm = pre.bm, n0 = pre.n0, n_last = pre.n_last;
  if (t == 0) { red[0] = red[1] = red[2] = 0; sel[0] = 0ull; sel[1] = 0ull; *n_live = 0u; }
  if (t < 128) l_mask[t] = 0ull;
  if (t < 64) { h_gt[t] = 0ull; h_eq[t] = 0ull; }
  __syncthreads();
  const long long cp = bm < n_last ? bm : n_last;
  if (head) { l_lb[t] = (int32_t)lb; l_cp[t] = (int32_t)cp; }
  const int h = mine ? t / Gp : 0, g = mine ? t - h * Gp : 0;
  if (mine) {
    l_kn[t] = vk;
    l_cu[t] = vc;
    if (vv) atomicOr(&l_mask[h * words + (g >> 6)], 1ull << (g & 63));
  }
  // minimum retention and units on offer are sums over heads (the segments of a head tile
  // (max(b_min, first knot), cap]): wave 0, 16-bit pieces cannot overflow a lane
  if (wave == 0) {
    const bool head_bad = head && (lb < 0 || lb > cp);
    const long long from = lb > n0 ? lb : n0;
    const unsigned offer = head && !head_bad && cp > from ? (unsigned)(cp - from) : 0u;
    const unsigned keep = head && !head_bad ? (unsigned)lb : 0u;
    const unsigned m_lo = wave_reduce_to_last(keep & 0xFFFFu, 0u, add), m_hi = wave_reduce_to_last(keep >> 16, 0u, add);
    const unsigned w_lo = wave_reduce_to_last(offer & 0xFFFFu, 0u, add), w_hi = wave_reduce_to_last(offer >> 16, 0u, add);
    const unsigned long long any_bad = __ballot(head_bad);
    if (lane == 63) {
      red[0] = (long long)(((unsigned long long)m_hi << 16) + m_lo);
      red[1] = (long long)(((unsigned long long)w_hi << 16) + w_lo);
      red[2] = any_bad ? 1 : 0;
    }
  }
  __syncthreads();
  // one segment per vertex (to the next vertex), clipped to (b_min, cap]; the live ones are listed
  {
    unsigned w = 0;
    unsigned long long key = 0;
    const unsigned long long* mk = l_mask + h * words;
    if (mine && g < Gp - 1 && ((mk[g >> 6] >> (g & 63)) & 1ull)) {
      int c = g + 1, wd = c >> 6;            // next vertex; the last knot is always one
      unsigned long long m = mk[wd] & (~0ull << (c & 63));
      while (m == 0ull && wd + 1 < words) m = mk[++wd];
      c = m ? wd * 64 + __ffsll((long long)m) - 1 : Gp - 1;
      const long long na = vk, nb = l_kn[h * Gp + c];
      const double ua = (double)vc, ub = (double)l_cu[h * Gp + c];
      const long long hlb = l_lb[h], hcp = l_cp[h];
      const long long lo = max(na, hlb), hi = min(nb, hcp);
      w = hi > lo ? (unsigned)(hi - lo) : 0u;
      key = gain_key((ub - ua) / (double)(nb - na));
    }
    const unsigned long long live = __ballot(w != 0u);
    if (live) {
      unsigned at = 0;
      const int leader = __ffsll((long long)live) - 1;
      if (lane == leader) at = atomicAdd(n_live, (unsigned)__popcll(live));
      at = (unsigned)__shfl((int)at, leader) + (unsigned)__popcll(live & ((1ull << lane) - 1ull));
      if (w) { live_key[at] = key; live_w[at] = w; live_h[at] = (unsigned short)h; }
    }
  }
  __syncthreads();
  const long long R = io.B[p] - red[0];
  const bool infeasible = red[2] != 0 || R < 0 || R > red[1];
  const bool active = !infeasible && R > 0;
  const int n = (int)*n_live;
  // threshold gain g*: W(> g*) < R <= W(>= g*), by ranking each live segment against all; a
  // power-of-two group of lanes shares one segment's ranking
  if (active) {
    int share = 1;
    while (share < 64 && n * share * 2 <= 1024) share *= 2;
    const int seg = t / share, sub = t % share;
    const bool have = seg < n;
    const unsigned long long me = have ? live_key[seg] : 0ull;
    unsigned long long w_gt = 0, w_eq = 0;
    if (have) {
#pragma unroll 4
      for (int j = sub; j < n; j += share) {
        const unsigned long long kj = live_key[j];
        const unsigned long long wj = live_w[j];
        w_gt += kj > me ? wj : 0ull;
        w_eq += kj == me ? wj : 0ull;
      }
    }
    for (int o = 1; o < share; o <<= 1) {
      w_gt += (unsigned long long)shfl_xor_i64((long long)w_gt, o);
      w_eq += (unsigned long long)shfl_xor_i64((long long)w_eq, o);
    }
    if (have && sub == 0 && w_gt < (unsigned long long)R && (unsigned long long)R <= w_gt + w_eq) {
      sel[0] = me;
      sel[1] = (unsigned long long)R - w_gt;
    }
  }
  __syncthreads();
  const unsigned long long kstar = sel[0];
  const long long rem = active ? (long long)sel[1] : 0;
  if (active && t < n) {
    const unsigned long long me = live_key[t];
    if (me > kstar) atomicAdd(&h_gt[live_h[t]], (unsigned long long)live_w[t]);
    else if (me == kstar) atomicAdd(&h_eq[live_h[t]], (unsigned long long)live_w[t]);
  }
  __syncthreads();
  // budgets: everything above g*, the units at g* in head order
  if (head) {
    long long eq_before = 0;
    for (int h2 = 0; h2 < t; ++h2) eq_before += (long long)h_eq[h2];
    const long long eq = (long long)h_eq[t];
    long long take = rem - eq_before;
    take = take < 0 ? 0 : (take > eq ? eq : take);
    const int32_t b = (int32_t)(lb + (active ? (long long)h_gt[t] + take : 0));
    if (write_out) io.budgets[hbase + t] = b;
    if (budgets_lds) budgets_lds[t] = b;
  }
  if (t == 0 && write_out) io.status[p] = infeasible ? LUKV_ST_INFEASIBLE : 0;
}

// whether alloc_phase_b_small takes the problem (by a workgroup of 1024 threads)
__host__ __device__ inline bool alloc_small_ok(int n_heads, int n_grid) {
  return n_heads <= 64 && n_heads * n_grid <= 1024;
}

// Phase B for problem p (after phase A's flags are visible); lds: scratch of lds_bytes, free
// for this call.
__device__ inline void alloc_phase_b(const AllocIO& io, int p, char* lds, int lds_bytes) {
  const int words = (io.n_grid + 63) / 64;
  if (blockDim.x == 1024 && lds_bytes >= 32768 && alloc_small_ok(io.n_heads, io.n_grid))
    alloc_phase_b_small(io, p, lds, alloc_small_load(io, p), nullptr, true);
  else if (blockDim.x == 1024 && lds_bytes >= kAllocLdsBytes && io.n_heads <= 1024 && io.n_heads * words <= 1024)
    alloc_phase_b_mid(io, p, lds);
  else
    alloc_phase_b_generic(io, p, lds, lds_bytes);
}

}  // namespace lukv

#pragma clang fp contract(fast)
